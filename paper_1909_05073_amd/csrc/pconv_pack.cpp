// Host side of pconv_pack: layer-wise information extraction, filter kernel reorder and compact
// weight storage (paper, "Compiler-assisted DNN Inference Framework").  Integer work only; the
// result is a deterministic function of the inputs.
#include <algorithm>
#include <cstring>
#include <numeric>

#include "pconv_internal.h"
#include "pconv_tiled_codes.h"

namespace pconv {

namespace {

// fp32 -> bf16 bit pattern, round to nearest, ties to even; NaNs stay quiet NaNs.
inline uint16_t bf16_rne(uint32_t u)
{
    const uint32_t exp_all_ones = 0x7F800000u;
    if ((u & exp_all_ones) == exp_all_ones && (u << 9) != 0) return uint16_t((u >> 16) | 0x40u);
    const uint32_t round_bias = 0x7FFFu + ((u >> 16) & 1u);
    return uint16_t((u + round_bias) >> 16);
}

}  // namespace

int build_canonical(const float *w, const uint8_t *pid, const uint8_t *conn, const uint16_t *table,
                    int np, int c_out, int c_in, int wdtype, Canonical &out)
{
    // ---- validation ------------------------------------------------------------------
    for (int p = 0; p < np; ++p)
        if (table[p] == 0 || table[p] > 0x1FF) {
            set_error("pconv_pack: table[" + std::to_string(p) + "] must be a non-zero 9-bit mask");
            return PCONV_INVALID_ARG;
        }
    const size_t fc = size_t(c_out) * c_in;
    for (size_t e = 0; e < fc; ++e)
        if (conn[e] && pid[e] >= np) {
            set_error("pconv_pack: pattern_id " + std::to_string(int(pid[e])) + " of kept kernel (f=" +
                      std::to_string(e / c_in) + ", c=" + std::to_string(e % c_in) +
                      ") is outside the pattern table");
            return PCONV_INVALID_ARG;
        }

    // ---- layer-wise information extraction: per-filter kernel count and pattern histogram
    std::vector<uint32_t> hist(size_t(c_out) * np, 0), kcnt(c_out, 0);
    for (int f = 0; f < c_out; ++f) {
        const uint8_t *cr = conn + size_t(f) * c_in, *pr = pid + size_t(f) * c_in;
        for (int c = 0; c < c_in; ++c)
            if (cr[c]) { ++kcnt[f]; ++hist[size_t(f) * np + pr[c]]; }
    }

    // ---- filter reorder: similar filters adjacent.  Key: kept count, then the histogram
    // compared pattern by pattern, larger first; the filter index breaks ties.
    std::vector<int> order(c_out);
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int a, int b) {
        if (kcnt[a] != kcnt[b]) return kcnt[a] > kcnt[b];
        const uint32_t *ha = &hist[size_t(a) * np], *hb = &hist[size_t(b) * np];
        if (!std::equal(ha, ha + np, hb)) return std::lexicographical_compare(hb, hb + np, ha, ha + np);
        return a < b;
    });

    // ---- kernel reorder inside a filter (pattern, then channel) + compact storage --------
    uint64_t K = 0, nnz = 0;
    int pop[PCONV_MAX_PATTERNS];
    for (int p = 0; p < np; ++p) pop[p] = __builtin_popcount(table[p]);
    for (int f = 0; f < c_out; ++f) {
        K += kcnt[f];
        for (int p = 0; p < np; ++p) nnz += uint64_t(hist[size_t(f) * np + p]) * pop[p];
    }
    if (nnz >= (1ull << 32)) { set_error("pconv_pack: more than 2^32 stored weights"); return PCONV_INVALID_ARG; }

    out.perm.resize(c_out);
    out.row_ptr.resize(size_t(c_out) + 1);
    out.pat_cnt.resize(size_t(c_out) * np);
    out.cin.resize(K);
    out.pat.resize(K);
    out.val_ptr.resize(K + 1);
    out.vals_bits.resize(nnz);

    uint32_t k = 0, v = 0;
    std::vector<uint32_t> start(np + 1);
    for (int i = 0; i < c_out; ++i) {
        const int f = order[i];
        out.perm[i] = uint16_t(f);
        out.row_ptr[i] = k;
        // counting sort by pattern; scanning channels in ascending order keeps (pattern, c) order
        start[0] = k;
        for (int p = 0; p < np; ++p) {
            out.pat_cnt[size_t(i) * np + p] = uint16_t(hist[size_t(f) * np + p]);
            start[p + 1] = start[p] + hist[size_t(f) * np + p];
        }
        const uint8_t *cr = conn + size_t(f) * c_in, *pr = pid + size_t(f) * c_in;
        for (int c = 0; c < c_in; ++c)
            if (cr[c]) {
                const uint32_t at = start[pr[c]]++;
                out.cin[at] = uint16_t(c);
                out.pat[at] = pr[c];
            }
        k += kcnt[f];
        // gather kept taps, kernel by kernel in the new order
        for (uint32_t q = out.row_ptr[i]; q < k; ++q) {
            out.val_ptr[q] = v;
            const float *src = w + (size_t(f) * c_in + out.cin[q]) * 9;
            const unsigned mask = table[out.pat[q]];
            for (int t = 0; t < 9; ++t)
                if (mask & (1u << t)) {
                    uint32_t bits;
                    std::memcpy(&bits, src + t, 4);
                    out.vals_bits[v++] = (wdtype == PCONV_BF16) ? uint32_t(bf16_rne(bits)) << 16 : bits;
                }
        }
    }
    out.row_ptr[c_out] = k;
    out.val_ptr[K] = v;
    return PCONV_OK;
}

// ---- stream of the register-tiled kernel ----------------------------------------------
//
// Workload balance (paper: the reorder exists so that threads get similar work).  Here a wave
// runs the kernels of its kTileFB filters one after another, so what must be equal across
// waves is the SUM of their kernel counts: the filters, already sorted by kernel count, are
// dealt to the blocks in serpentine order (0..NB-1, NB-1..0, ...), which gives every block
// one filter from each slice of the sorted list; a local search then evens the counts out
// chunk by chunk (see below).
void build_tiled_stream(const Canonical &cn, const uint16_t *table, int np, int c_out, int c_in,
                        TiledStream &out)
{
    const int FB = kTileFB;
    const int nb = (c_out + FB - 1) / FB;
    const int cpad = (c_in + kTileCH - 1) / kTileCH * kTileCH;
    out.num_blocks = nb;
    out.row_len = cpad + 1;
    out.slot_filter.assign(size_t(nb) * FB, -1);
    std::vector<int> slot_pos(size_t(nb) * FB, -1);          // position in the sorted order
    for (int i = 0; i < c_out; ++i) {
        const int round = i / nb, idx = i % nb;
        const int blk = (round & 1) ? nb - 1 - idx : idx;
        out.slot_filter[size_t(blk) * FB + round] = cn.perm[i];
        slot_pos[size_t(blk) * FB + round] = i;
    }

    // split every pattern into disjoint codes: largest compiled sub-mask first
    struct Piece { int code; int tap_rank[4]; int ntaps; };   // tap_rank: index into the kernel's stored weights
    std::vector<std::vector<Piece>> pieces(np);
    for (int p = 0; p < np; ++p) {
        unsigned left = table[p];
        while (left) {
            int best = -1, best_pop = 0;
            for (int cidx = 0; cidx < kNumCodes; ++cidx) {
                const unsigned m = kCodeMask[cidx];
                if ((m & left) == m && __builtin_popcount(m) > best_pop) { best = cidx; best_pop = __builtin_popcount(m); }
            }
            Piece pc{best, {0, 0, 0, 0}, 0};
            for (int t = 0; t < 9; ++t)
                if (kCodeMask[best] & (1u << t))
                    pc.tap_rank[pc.ntaps++] = __builtin_popcount(unsigned(table[p]) & ((1u << t) - 1u));
            pieces[p].push_back(pc);
            left &= ~unsigned(kCodeMask[best]);
        }
    }

    // Second step of the balance: the waves of a workgroup walk the input channels chunk by chunk
    // (kTileCH channels) and may drift at most a chunk apart, so their record counts should agree
    // chunk by chunk, not only in total.  Within every group of kTileWaves blocks (the filters of
    // one workgroup) filters are swapped between blocks while that lowers
    //     sum over blocks b [ sum over chunks j of L(b, j)^2  +  (sum over chunks j of L(b, j))^2 / J ],
    // L(b, j) = records of block b in chunk j: a plain local search, deterministic, a few passes.
    {
        const int J = cpad / kTileCH;
        const int GW = kTileWaves;
        std::vector<int> cnt;                                 // [slots of the group][J] records of the slot's filter
        std::vector<int64_t> load, total;
        for (int g0 = 0; g0 < nb; g0 += GW) {
            const int gb = std::min(GW, nb - g0), gs = gb * FB;
            cnt.assign(size_t(gs) * J, 0);
            for (int sl = 0; sl < gs; ++sl) {
                const int pos = slot_pos[size_t(g0) * FB + sl];
                if (pos < 0) continue;
                for (uint32_t k = cn.row_ptr[pos]; k < cn.row_ptr[pos + 1]; ++k)
                    cnt[size_t(sl) * J + cn.cin[k] / kTileCH] += int(pieces[cn.pat[k]].size());
            }
            load.assign(size_t(gb) * J, 0); total.assign(gb, 0);
            for (int sl = 0; sl < gs; ++sl)
                for (int j = 0; j < J; ++j) { load[size_t(sl / FB) * J + j] += cnt[size_t(sl) * J + j]; total[sl / FB] += cnt[size_t(sl) * J + j]; }
            for (int pass = 0; pass < 16; ++pass) {
                bool improved = false;
                for (int sa = 0; sa < gs; ++sa)
                    for (int sb = sa + 1; sb < gs; ++sb) {
                        const int ba = sa / FB, bb = sb / FB;
                        if (ba == bb) continue;
                        // cost change if the filters in slots sa and sb trade places (times J, to stay in integers)
                        int64_t delta = 0, ta = 0, tb = 0;
                        for (int j = 0; j < J; ++j) {
                            const int64_t d = int64_t(cnt[size_t(sb) * J + j]) - cnt[size_t(sa) * J + j];   // block a gains d, block b loses d
                            const int64_t la = load[size_t(ba) * J + j], lb = load[size_t(bb) * J + j];
                            delta += (la + d) * (la + d) - la * la + (lb - d) * (lb - d) - lb * lb;
                            ta += d;
                        }
                        tb = -ta;
                        delta = delta * J + (total[ba] + ta) * (total[ba] + ta) - total[ba] * total[ba]
                                          + (total[bb] + tb) * (total[bb] + tb) - total[bb] * total[bb];
                        if (delta >= 0) continue;
                        for (int j = 0; j < J; ++j) {
                            const int64_t d = int64_t(cnt[size_t(sb) * J + j]) - cnt[size_t(sa) * J + j];
                            load[size_t(ba) * J + j] += d; load[size_t(bb) * J + j] -= d;
                            std::swap(cnt[size_t(sa) * J + j], cnt[size_t(sb) * J + j]);
                        }
                        total[ba] += ta; total[bb] += tb;
                        std::swap(out.slot_filter[size_t(g0) * FB + sa], out.slot_filter[size_t(g0) * FB + sb]);
                        std::swap(slot_pos[size_t(g0) * FB + sa], slot_pos[size_t(g0) * FB + sb]);
                        improved = true;
                    }
                if (!improved) break;
            }
        }
    }

    out.chan_ptr.assign(size_t(nb) * out.row_len, 0);
    out.meta.clear();
    out.w4.clear();
    std::vector<std::vector<int32_t>> by_slot(FB, std::vector<int32_t>(size_t(c_in), -1));
    for (int b = 0; b < nb; ++b) {
        for (int s = 0; s < FB; ++s) {
            std::fill(by_slot[s].begin(), by_slot[s].end(), -1);
            const int pos = slot_pos[size_t(b) * FB + s];
            if (pos < 0) continue;
            for (uint32_t k = cn.row_ptr[pos]; k < cn.row_ptr[pos + 1]; ++k) by_slot[s][cn.cin[k]] = int32_t(k);
        }
        uint32_t *row = &out.chan_ptr[size_t(b) * out.row_len];
        for (int c = 0; c < c_in; ++c) {
            row[c] = uint32_t(out.meta.size());
            bool first = true;
            for (int s = 0; s < FB; ++s) {
                const int32_t k = by_slot[s][c];
                if (k < 0) continue;
                for (const Piece &pc : pieces[cn.pat[k]]) {
                    out.meta.push_back(uint32_t(s * kNumCodes + pc.code) << kMetaCaseShift | uint32_t(c % kTileCH) |
                                       (first ? kMetaFirstOfChannel : 0u));
                    first = false;
                    for (int j = 0; j < 4; ++j) {
                        float v = 0.0f;
                        if (j < pc.ntaps) std::memcpy(&v, &cn.vals_bits[cn.val_ptr[k] + pc.tap_rank[j]], 4);
                        out.w4.push_back(v);
                    }
                }
            }
        }
        for (int c = c_in; c <= cpad; ++c) row[c] = uint32_t(out.meta.size());
    }
    // padding: the kernel asks for the words of records k+1 and k+2 while it executes record k
    for (int j = 0; j < 3; ++j) out.meta.push_back(0u);
    for (int j = 0; j < 4; ++j) out.w4.push_back(0.0f);
}

// ---- dense per-tap matrices of the matrix-core kernel -----------------------------------
void build_dense_taps(const Canonical &cn, const uint16_t *table, int c_out, int c_in,
                      std::vector<uint16_t> &wd, std::vector<uint32_t> &nz)
{
    const int fpad = (c_out + 31) / 32 * 32, cb32 = (c_in + 31) / 32, cb16 = cb32 * 2;
    wd.assign(size_t(9) * cb16 * fpad * 16, 0);
    nz.assign(size_t(cb32) * (fpad / 32), 0u);
    for (int i = 0; i < c_out; ++i) {
        const int f = cn.perm[i];
        for (uint32_t k = cn.row_ptr[i]; k < cn.row_ptr[i + 1]; ++k) {
            const int c = cn.cin[k];
            const unsigned mask = table[cn.pat[k]];
            uint32_t v = cn.val_ptr[k];
            for (int t = 0; t < 9; ++t)
                if (mask & (1u << t)) {
                    wd[((size_t(t) * cb16 + c / 16) * fpad + f) * 16 + c % 16] = uint16_t(cn.vals_bits[v++] >> 16);
                    nz[size_t(c / 32) * (fpad / 32) + f / 32] |= 1u << (2 * t + (c / 16) % 2);
                }
        }
    }
}

// ---- projection of dense weights onto the PCONV constraints ------------------------------
//
// Pattern assignment: the table mask under which a kernel keeps the most energy (sum of squares of
// the kept taps; the first such mask among equals).  Connectivity: the `keep` kernels that keep the
// most energy under their mask survive (the lower (f, c) among equals).  Energies are accumulated in
// double over the taps in ascending order, so equal inputs decide equally everywhere.
int project_weights(const float *w, const uint16_t *table, int np, int c_out, int c_in, int64_t keep,
                    uint8_t *pattern_id, uint8_t *conn)
{
    const size_t total = size_t(c_out) * c_in;
    std::vector<double> energy(total);
    for (size_t k = 0; k < total; ++k) {
        double sq[9];
        for (int t = 0; t < 9; ++t) sq[t] = double(w[9 * k + t]) * double(w[9 * k + t]);
        int arg = 0;
        double top = -1.0;
        for (int p = 0; p < np; ++p) {
            double e = 0.0;
            for (unsigned m = table[p], t = 0; m; m >>= 1, ++t)
                if (m & 1u) e += sq[t];
            if (e > top) { top = e; arg = p; }
        }
        pattern_id[k] = uint8_t(arg);
        energy[k] = top;
    }
    std::fill(conn, conn + total, uint8_t(0));
    if (keep <= 0) return PCONV_OK;
    std::vector<uint32_t> order(total);
    std::iota(order.begin(), order.end(), 0u);
    const size_t kk = std::min<size_t>(size_t(keep), total);
    // (a strict order: energy descending, then index ascending - the kept set does not depend on the algorithm)
    auto before = [&](uint32_t a, uint32_t b) { return energy[a] != energy[b] ? energy[a] > energy[b] : a < b; };
    if (kk < total) std::nth_element(order.begin(), order.begin() + kk, order.end(), before);
    for (size_t i = 0; i < kk; ++i) conn[order[i]] = 1;
    return PCONV_OK;
}

}  // namespace pconv
