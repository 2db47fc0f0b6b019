// Host-only logic of the library (layouts, chunk plan, metadata builder, validation) run on exact-size buffers
// under AddressSanitizer / UBSan.  Built and run by tests/test_host_asan.py; no GPU involved.
#include <cstdio>
#include <cstring>
#include <cstdint>
#include <cstdlib>
#include <vector>

#include "hr_internal.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main() {
    // chunk plan of mixed lengths, metadata written into a buffer of exactly the computed size
    std::vector<int32_t> lens = {270, 4, 64, 65, 128, 2112, 1};
    for (int chunk : {32, 64}) {
        hr::ChunkPlan cp = hr::make_chunk_plan((int64_t)lens.size(), lens.data(), chunk);
        hr::MetaLayout ml = hr::make_meta_layout(cp.n_chunks, cp.T, cp.pt_stride, (int64_t)lens.size(), 10);
        std::vector<int32_t> meta(ml.total, -7), toks(cp.T, 1);
        hr::fill_meta(meta.data(), ml, cp.n_chunks, cp.prefix_lens.data(), cp.new_lens.data(), toks.data(), cp.page_table.data(),
                      cp.pt_stride, cp.out_row.data(), (int64_t)lens.size());
        int64_t total = 0;
        for (int32_t l : lens) total += l;
        CHECK(cp.T == total);
        CHECK(meta[ml.cu + cp.n_chunks] == total);
        // every chunk starts on a 32-slot boundary and a sequence's pages are contiguous
        int64_t ci = 0;
        for (size_t s = 0; s < lens.size(); ++s) {
            for (int64_t off = 0; off < lens[s]; off += chunk, ++ci) {
                CHECK(meta[ml.new_cu + ci] % 32 == 0);
                CHECK(meta[ml.new_cu + ci] == cp.first_page[s] * 16 + off);
                CHECK(meta[ml.prefix_len + ci] == off);
                for (int64_t pg = 0; pg < off / 16; ++pg) CHECK(meta[ml.page_table + ci * cp.pt_stride + pg] == cp.first_page[s] + pg);
            }
            CHECK(meta[ml.out_row + s] == meta[ml.cu + ci] - 1);
        }
    }
    // scoring layout: positions continue after the document, slots are 32-aligned per pair
    std::vector<int32_t> dl = {100, 0, 17}, ql = {5, 1, 33}, pt(3 * 7, 3), tk(39, 2);
    hr::MetaLayout m2 = hr::make_meta_layout(3, 39, 7);
    std::vector<int32_t> meta2(m2.total);
    hr::fill_meta(meta2.data(), m2, 3, dl.data(), ql.data(), tk.data(), pt.data(), 7);
    CHECK(meta2[m2.tok_pos + 0] == 100 && meta2[m2.tok_pos + 4] == 104 && meta2[m2.tok_pos + 5] == 0 && meta2[m2.tok_pos + 6] == 17);
    CHECK(meta2[m2.new_cu + 0] == 0 && meta2[m2.new_cu + 1] == 32 && meta2[m2.new_cu + 2] == 64 && meta2[m2.new_cu + 3] == 128);
    CHECK(meta2[m2.out_row + 0] == 4 && meta2[m2.out_row + 1] == 5 && meta2[m2.out_row + 2] == 38);
    // group plan: pairs with identical page-table rows and lengths share a group up to the block capacity; every
    // block and every 32-key sub-tile of every pair appears exactly once; groups come heaviest first
    {
        const int g = 7, cap = 16, stride = 4;
        // docs: A = pages {3, 9}, len 30; B = pages {5}, len 16; pair 6 has A's first page but another second page
        std::vector<int32_t> gd = {30, 16, 30, 0, 30, 16, 30, 0, 30}, gq = {40, 8, 33, 5, 64, 1, 9, 5, 20};
        std::vector<int32_t> gpt = {3, 9, -1, -1, 5, -1, -1, -1, 3, 9, -1, -1, -1, -1, -1, -1, 3, 9, -1, -1, 5, -1, -1, -1,
                                    3, 8, -1, -1, -1, -1, -1, -1, 3, 9, -1, -1};
        const int64_t n = (int64_t)gd.size();
        int64_t Tq = 0;
        for (int32_t v : gq) Tq += v;
        hr::GroupPlan gp = hr::make_group_plan(n, gd.data(), gq.data(), gpt.data(), stride, g, cap);
        CHECK(gp.ints() <= hr::group_plan_ints_bound(n, Tq, g));
        std::vector<int32_t> flat(gp.ints(), -7);
        hr::store_group_plan(gp, flat.data());
        CHECK(flat[0] == gp.p0[0] && flat.back() == gp.sub_key0.back());
        CHECK(gp.shared && gp.max_blocks <= cap);
        CHECK((int)gp.blk_cu.size() == gp.n_groups + 1 && (int)gp.sub_cu.size() == gp.n_groups + 1);
        std::vector<int> blocks_seen(n, 0), subs_seen(n, 0), group_of(n, -1);
        int64_t prev_cost = INT64_MAX;
        std::vector<int64_t> new_page(n);
        int64_t slot = 0;
        for (int64_t p = 0; p < n; ++p) { new_page[p] = slot / 16; slot += (gq[p] + 31) / 32 * 32; }
        for (int gi = 0; gi < gp.n_groups; ++gi) {
            const int32_t lead = gp.p0[gi];
            const int nb = gp.blk_cu[gi + 1] - gp.blk_cu[gi];
            CHECK(nb >= 1 && nb <= cap);
            const int64_t cost = ((int64_t)gd[lead] + 64) * nb;
            CHECK(cost <= prev_cost);
            prev_cost = cost;
            for (int b = gp.blk_cu[gi]; b < gp.blk_cu[gi + 1]; ++b) {
                const int32_t p = gp.blk_seq[b];
                CHECK(p >= 0 && p < n && gd[p] == gd[lead]);
                for (int pg = 0; pg < (gd[p] + 15) / 16; ++pg) CHECK(gpt[p * stride + pg] == gpt[lead * stride + pg]);
                CHECK(group_of[p] == -1 || group_of[p] == gi);
                group_of[p] = gi;
                CHECK(gp.blk_row0[b] == 32 * blocks_seen[p]);              // a pair's blocks in order, back to back
                CHECK(b == gp.blk_cu[gi] || gp.blk_seq[b - 1] == p || blocks_seen[p] == 0);
                ++blocks_seen[p];
            }
            for (int s = gp.sub_cu[gi]; s < gp.sub_cu[gi + 1]; ++s) {
                const int32_t p = gp.sub_seq[s];
                CHECK(group_of[p] == gi);
                CHECK(gp.sub_key0[s] == 32 * subs_seen[p] && gp.sub_page[s] == new_page[p] + 2 * subs_seen[p]);
                ++subs_seen[p];
            }
        }
        for (int64_t p = 0; p < n; ++p) {
            CHECK(blocks_seen[p] == (gq[p] * g + 31) / 32 && subs_seen[p] == (gq[p] + 31) / 32);
            if (gd[p] == 0) CHECK(gp.blk_cu[group_of[p] + 1] - gp.blk_cu[group_of[p]] == blocks_seen[p]);   // no document: alone
        }
        // A is shared by pairs 0, 2, 4, 8 (9 + 8 + 14 + 5 blocks): at least two groups; pair 6 is not with them
        CHECK(group_of[6] != group_of[0] && group_of[6] != group_of[2] && group_of[6] != group_of[4] && group_of[6] != group_of[8]);
        CHECK(group_of[1] == group_of[5]);
        CHECK(group_of[3] != group_of[7]);
        // nothing shared: every pair alone
        std::vector<int32_t> upt = {1, 2, 3};
        std::vector<int32_t> ud = {16, 16, 16}, uq = {4, 4, 4};
        hr::GroupPlan up = hr::make_group_plan(3, ud.data(), uq.data(), upt.data(), 1, g, cap);
        CHECK(!up.shared && up.n_groups == 3 && up.max_blocks == 1);
        CHECK(!up.uneven && gp.uneven);
        // scarce work items: sequences are cut into pieces of at most 4 blocks; every (sequence, block) exactly once, and
        // every group lists the own keys of each of its sequences exactly once
        hr::GroupPlan cp4 = hr::make_group_plan(n, gd.data(), gq.data(), gpt.data(), stride, g, 4, true);
        CHECK(cp4.cut && cp4.max_blocks <= 4 && cp4.ints() <= hr::group_plan_ints_bound(n, Tq, g));
        std::vector<std::vector<char>> seen(n);
        for (int64_t p = 0; p < n; ++p) seen[p].assign((gq[p] * g + 31) / 32, 0);
        for (int gi = 0; gi < cp4.n_groups; ++gi) {
            std::vector<int> subs_in_group(n, 0), blocks_in_group(n, 0);
            for (int b = cp4.blk_cu[gi]; b < cp4.blk_cu[gi + 1]; ++b) {
                const int32_t p = cp4.blk_seq[b];
                CHECK(cp4.blk_row0[b] % 32 == 0 && cp4.blk_row0[b] / 32 < (int)seen[p].size() && !seen[p][cp4.blk_row0[b] / 32]);
                seen[p][cp4.blk_row0[b] / 32] = 1;
                CHECK(gd[p] == gd[cp4.p0[gi]]);
                ++blocks_in_group[p];
            }
            for (int sidx = cp4.sub_cu[gi]; sidx < cp4.sub_cu[gi + 1]; ++sidx) {
                const int32_t p = cp4.sub_seq[sidx];
                CHECK(cp4.sub_key0[sidx] == 32 * subs_in_group[p] && cp4.sub_page[sidx] == new_page[p] + 2 * subs_in_group[p]);
                ++subs_in_group[p];
            }
            for (int64_t p = 0; p < n; ++p) CHECK(subs_in_group[p] == (blocks_in_group[p] ? (gq[p] + 31) / 32 : 0));
        }
        for (int64_t p = 0; p < n; ++p)
            for (char c : seen[p]) CHECK(c == 1);
        // many sequences of up to 16 blocks cut into pieces of at most 8 (128-wide heads): fits the room reserved for a plan
        {
            const int64_t nn = 300;
            const int g8 = 8;
            std::vector<int32_t> md(nn), mq(nn), mpt(nn);
            int64_t Tm = 0;
            for (int64_t p = 0; p < nn; ++p) {
                md[p] = 16;
                mq[p] = 1 + (int32_t)((p * 37) % 64);
                mpt[p] = (int32_t)(p % 7);                   // a few shared first pages (same length: shared documents)
                Tm += mq[p];
            }
            hr::GroupPlan cp8 = hr::make_group_plan(nn, md.data(), mq.data(), mpt.data(), 1, g8, 8, true);
            CHECK(cp8.cut && cp8.max_blocks <= 8 && cp8.ints() <= hr::group_plan_ints_bound(nn, Tm, g8));
            std::vector<int> blocks(nn, 0);
            for (size_t b = 0; b < cp8.blk_seq.size(); ++b) ++blocks[cp8.blk_seq[b]];
            for (int64_t p = 0; p < nn; ++p) CHECK(blocks[p] == (mq[p] * g8 + 31) / 32);
        }
        std::vector<int32_t> rd = {16, 48, 32};                   // nothing shared, lengths differ: heaviest first
        hr::GroupPlan rp = hr::make_group_plan(3, rd.data(), uq.data(), upt.data(), 1, g, cap);
        CHECK(!rp.shared && rp.uneven && rp.p0[0] == 1 && rp.p0[1] == 2 && rp.p0[2] == 0);
    }
    // a call cut in two halves: the two carvings fit the whole call's workspace plus the 1 MB the size query adds
    {
        hr_model_cfg mcs[2] = {{24, 896, 14, 2, 64, 4864, 1000, 1, 2, HR_BF16, 1e6f, 1e-6f}, {32, 4096, 32, 8, 128, 14336, 1000, 1, 2, HR_BF16, 5e5f, 1e-5f}};
        unsigned rs = 12345u;
        auto rnd = [&](unsigned n) { rs = rs * 1664525u + 1013904223u; return (rs >> 8) % n; };
        for (int it = 0; it < 400; ++it) {
            const hr_model_cfg& mc2 = mcs[it & 1];
            const int g2 = mc2.n_q_heads / mc2.n_kv_heads;
            const int64_t n = 2 + rnd(3000), T = n + rnd(40000), stride = 1 + rnd(130);
            const int64_t na = 1 + rnd((unsigned)(n - 1)), Ta = na + rnd((unsigned)(T - n + 1));       // Ta >= na, Tb >= nb
            const int64_t nb = n - na, Tb = T - Ta;
            if (Tb < nb) continue;
            const size_t whole = hr::make_workspace(mc2, n, T, stride, false, -1, 0, (int64_t)hr::group_plan_ints_bound(n, T, g2)).total;
            const size_t a_part = hr::make_workspace(mc2, na, Ta, stride, false, -1, 0, (int64_t)hr::group_plan_ints_bound(na, Ta, g2)).total;
            const size_t b_part = hr::make_workspace(mc2, nb, Tb, stride, false, -1, 0, (int64_t)hr::group_plan_ints_bound(nb, Tb, g2)).total;
            CHECK(a_part + b_part <= whole + (1 << 20));
        }
    }
    // pool bookkeeping and validation paths
    hr_pool_cfg pc{2, 2, 64, 16, 8, HR_BF16};
    hr_pool* pool = nullptr;
    CHECK(hr_kv_pool_create(&pc, (void*)0x1000, hr_kv_pool_bytes(&pc), &pool) == HR_OK);
    int32_t ids[3] = {1, 5, 1};
    CHECK(hr::pool_check_write(pool, 40, ids) == HR_ERR_PAGE_DUP);
    ids[2] = 7;
    CHECK(hr::pool_check_write(pool, 40, ids) == HR_OK);
    CHECK(hr::pool_check_read(pool, 40, ids) == HR_ERR_TABLE_SHORT);
    hr::pool_mark(pool, ids, 3, hr::PAGE_USED);
    CHECK(hr_kv_pool_free_pages(pool) == 5);
    CHECK(hr::pool_check_read(pool, 40, ids) == HR_OK);
    CHECK(hr::pool_check_read(pool, 0, ids) == HR_ERR_LEN_RANGE);
    hr_model_cfg mc{2, 128, 4, 2, 64, 256, 100, 1, 2, HR_BF16, 10000.f, 1e-6f};
    int32_t table[2 * 3] = {1, 5, 7, 1, 5, -1};
    int32_t dls[2] = {40, 32}, qls[2] = {3, 2}, qt[5] = {1, 2, 3, 4, 99};
    int64_t T = 0;
    CHECK(hr::score_check_args(mc, pool, 2, table, 3, dls, qt, qls, 1 << 20, &T) == HR_OK && T == 5);
    qt[4] = 100;
    CHECK(hr::score_check_args(mc, pool, 2, table, 3, dls, qt, qls, 1 << 20, &T) == HR_ERR_TOKEN_RANGE);
    dls[1] = 48;
    CHECK(hr::score_check_args(mc, pool, 2, table, 3, dls, qt, qls, 1 << 20, &T) == HR_ERR_TABLE_SHORT);
    hr_kv_pool_destroy(pool);

    // tile shape choice: the chosen shape is the cheapest of the model, the tall tile only where allowed and only where it
    // saves rounds, the fill of the rounds lies in (0, 1]; the cases the design names come out as stated
    {
        auto rounds = [](int64_t tiles, int64_t slots) { return (tiles + slots - 1) / slots; };
        std::srand(7);
        for (int it = 0; it < 2000; ++it) {
            const int64_t M = 1 + std::rand() % 120000;
            const int N = 64 * (1 + std::rand() % 480);
            const int cus = 8 * (1 + std::rand() % 40);
            const hr::TileChoice no_tall = hr::choose_gemm_tile(M, N, 128, false, cus);
            const hr::TileChoice any = hr::choose_gemm_tile(M, N, 128, true, cus);
            CHECK(no_tall != hr::TILE_TALL);
            if (any == hr::TILE_TALL) {
                const int64_t big = ((M + 255) / 256) * ((N + 255) / 256), tall = ((M + 319) / 320) * ((N + 255) / 256);
                CHECK(rounds(tall, cus) < rounds(big, cus));
            } else {
                CHECK(any == no_tall);
            }
            const double fill = hr::gemm_tile_fill(M, N, cus);
            CHECK(fill > 0.0 && fill <= 1.0);
        }
        CHECK(hr::choose_gemm_tile(20480, 896, 128, true, 256) == hr::TILE_TALL);      // 320 big tiles = 2 rounds, 256 tall = 1
        CHECK(hr::choose_gemm_tile(20480, 896, 128, false, 256) == hr::TILE_SMALL);     // 1120 small tiles in 3 rounds beat 2 big rounds
        CHECK(hr::gemm_tile_fill(20480, 896, 256) == 1.0);
        CHECK(hr::choose_gemm_tile(10240, 896, 128, true, 256) == hr::TILE_BIG);       // one round either way: the cheaper tile
        CHECK(hr::choose_gemm_tile(12800, 4096, 128, true, 256) == hr::TILE_TALL);     // 800 -> 640 tiles, 4 -> 3 rounds
        const double f8b = hr::gemm_tile_fill(12800, 4096, 256);
        CHECK(f8b > 0.83 && f8b < 0.84);                                               // 640 of 768 slots
        CHECK(hr::gemm_tile_fill(25600, 4096, 256) == 1.0);                            // 1280 tall tiles = 5 full rounds
    }
    {   // sequences with the same token string share first-layer rows: tables written into a layout of exactly the computed size
        // strings: A = {5, 6, 7}, B = {5, 6}, C = {9}; sequences A B A C B A C
        const std::vector<int32_t> lens = {3, 2, 3, 1, 2, 3, 1};
        const std::vector<int32_t> toks = {5, 6, 7, 5, 6, 5, 6, 7, 9, 5, 6, 5, 6, 7, 9};
        const int64_t n = (int64_t)lens.size(), T = (int64_t)toks.size();
        const hr::QueryShare qs = hr::make_query_share(n, lens.data(), toks.data());
        CHECK(qs.n_uniq == 6 && (int64_t)qs.rep_row.size() == 6 && (int64_t)qs.tok_src.size() == T);
        const std::vector<int32_t> want_rep = {0, 1, 2, 3, 4, 8};
        const std::vector<int32_t> want_src = {0, 1, 2, 3, 4, 0, 1, 2, 5, 3, 4, 0, 1, 2, 5};
        CHECK(qs.rep_row == want_rep && qs.tok_src == want_src);
        for (int64_t t = 0; t < T; ++t) CHECK(toks[qs.rep_row[qs.tok_src[t]]] == toks[t]);
        const hr::MetaLayout ml = hr::make_meta_layout(n, T, 4, -1, 0, 10, true);
        CHECK(ml.rep_row >= ml.tok_src + (size_t)T && ml.grp >= ml.rep_row + (size_t)T / 2 + 1 && ml.total >= ml.grp + 10);
        CHECK(qs.n_uniq * 2 <= T);                           // the tables fit the room the layout gives them
        std::vector<int32_t> meta(ml.total, -7);
        std::memcpy(meta.data() + ml.tok_src, qs.tok_src.data(), sizeof(int32_t) * qs.tok_src.size());
        std::memcpy(meta.data() + ml.rep_row, qs.rep_row.data(), sizeof(int32_t) * qs.rep_row.size());
        // equal hashes of different strings must not merge: same length, tokens differ in one place
        const std::vector<int32_t> l2 = {2, 2, 2};
        const std::vector<int32_t> t2 = {1, 2, 1, 3, 1, 2};
        const hr::QueryShare q2 = hr::make_query_share(3, l2.data(), t2.data());
        CHECK(q2.n_uniq == 4 && q2.tok_src[4] == 0 && q2.tok_src[5] == 1 && q2.tok_src[2] == 2);
        const hr::QueryShare q0 = hr::make_query_share(0, l2.data(), t2.data());
        CHECK(q0.n_uniq == 0 && q0.tok_src.empty());
        // workspace: the split form doubles the activation buffers, the shared form adds fp32 rows for half the tokens
        hr_model_cfg mc{2, 256, 4, 2, 64, 320, 500, 1, 2, HR_BF16, 10000.0f, 1e-6f};
        const hr::Workspace w0 = hr::make_workspace(mc, 4, 100, 3, false), w1 = hr::make_workspace(mc, 4, 100, 3, false, -1, 0, 0, true),
                            w2 = hr::make_workspace(mc, 4, 100, 3, false, -1, 0, 0, false, true);
        CHECK(w1.total > w0.total && w2.total > w0.total && w1.off_kvlo >= w1.off_v && w1.off_o > w1.off_kvlo && w0.off_o == w0.off_kvlo);
    }
    std::printf("host logic clean under sanitizers\n");
    return 0;
}
