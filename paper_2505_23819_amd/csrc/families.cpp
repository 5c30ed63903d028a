// Layout constructors and family tests: identity maps between labelled dims, blocked layouts
// (appendix, Proposition "Blocked layouts are linear layouts"), CDNA matrix-instruction tiles as
// products of identities (the pattern of the appendix's proof for `mma`), the legacy `mma` swizzle
// in closed form (Sec. 4.3, Def. "mma swizzling"), Def. "Distributed Layout", Def. "Memory Layout".
#include <vector>

#include "layout.hpp"

using f2::mat;
using f2::vec;
using ll::fail;

namespace {

bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }
int log2i(int x) { return 31 - __builtin_clz((unsigned)x); }

// Incremental builder: "the next k bits of label L go to the next k bits of dim D".
struct Builder {
    int n_dims;
    int dim_bits[LL_MAX_OUT_DIMS] = {};
    struct Piece { int label, dim, first, k; };
    std::vector<Piece> pieces;
    explicit Builder(int n) : n_dims(n) {}
    void add(int label, int dim, int k)
    {
        if (k <= 0) return;
        pieces.push_back({label, dim, dim_bits[dim], k});
        dim_bits[dim] += k;
    }
    ll_status finish(ll_layout **out) const
    {
        ll_out_dim odims[LL_MAX_OUT_DIMS];
        int shift[LL_MAX_OUT_DIMS], total = 0;
        for (int j = n_dims - 1; j >= 0; --j) {
            odims[j].nbits = dim_bits[j];
            shift[j] = total;
            total += dim_bits[j];
        }
        ll_in_dim idims[LL_MAX_IN_DIMS];
        int n_in = 0;
        mat cols;
        for (int label = LL_IN_REG; label <= LL_IN_OFFSET; ++label) {
            int bits = 0;
            for (const Piece &p : pieces)
                if (p.label == label)
                    for (int i = 0; i < p.k; ++i, ++bits) cols.push_back(vec(1) << (shift[p.dim] + p.first + i));
            if (bits > 0) {
                idims[n_in].label = label;
                idims[n_in].nbits = bits;
                ++n_in;
            }
        }
        if (n_in == 0) return fail(LL_ERR_INVALID_ARG, "the layout has no input bits");
        if ((int)cols.size() > LL_MAX_BITS || total > LL_MAX_BITS) return fail(LL_ERR_INVALID_ARG, "layout exceeds %d bits", LL_MAX_BITS);
        return ll::make_layout(idims, n_in, odims, n_dims, cols, out);
    }
};

ll_status check_out(ll_layout **out, int n_dims)
{
    if (!out) return fail(LL_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (n_dims < 1 || n_dims > LL_MAX_OUT_DIMS) return fail(LL_ERR_INVALID_ARG, "n_dims must be in [1, %d]", LL_MAX_OUT_DIMS);
    return LL_OK;
}

}  // namespace

extern "C" {

ll_status ll_layout_identity(int label, int dim, int k, int n_dims, ll_layout **out)
{
    try {
        if (ll_status st = check_out(out, n_dims); st != LL_OK) return st;
        if (label < LL_IN_REG || label > LL_IN_OFFSET) return fail(LL_ERR_INVALID_ARG, "unknown input label %d", label);
        if (dim < 0 || dim >= n_dims || k < 1 || k > LL_MAX_BITS) return fail(LL_ERR_INVALID_ARG, "bad dim %d or size %d", dim, k);
        Builder b(n_dims);
        b.add(label, dim, k);
        return b.finish(out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_identity: out of host memory");
    }
}

ll_status ll_layout_blocked(int n_dims, const int32_t *reg_bits, const int32_t *lane_bits, const int32_t *wave_bits,
                            const int32_t *order, ll_layout **out)
{
    try {
        if (ll_status st = check_out(out, n_dims); st != LL_OK) return st;
        if (!reg_bits || !lane_bits || !wave_bits || !order) return fail(LL_ERR_INVALID_ARG, "null argument");
        unsigned seen = 0;
        for (int i = 0; i < n_dims; ++i) {
            if (order[i] < 0 || order[i] >= n_dims || ((seen >> order[i]) & 1)) return fail(LL_ERR_INVALID_ARG, "order is not a permutation of the dims");
            seen |= 1u << order[i];
            if (reg_bits[i] < 0 || lane_bits[i] < 0 || wave_bits[i] < 0) return fail(LL_ERR_INVALID_ARG, "negative size");
        }
        // id_R^o x id_T^o x id_W^o: inside each resource the fastest dim takes the lowest bits, and in
        // every dim registers sit below lanes below waves
        Builder b(n_dims);
        const int32_t *per_label[3] = {reg_bits, lane_bits, wave_bits};
        for (int l = 0; l < 3; ++l)
            for (int i = 0; i < n_dims; ++i) b.add(LL_IN_REG + l, order[i], per_label[l][order[i]]);
        return b.finish(out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_blocked: out of host memory");
    }
}

ll_status ll_layout_mfma_accumulator(int m_bits, ll_layout **out)
{
    try {
        if (ll_status st = check_out(out, 2); st != LL_OK) return st;
        if (m_bits != 4 && m_bits != 5) return fail(LL_ERR_INVALID_ARG, "accumulator tiles are 16x16 (m_bits 4) or 32x32 (m_bits 5)");
        // a lane holds 4 consecutive rows of one column; lanes run along the columns, then over row
        // blocks; the remaining registers step over the rest of the rows
        Builder b(2);
        b.add(LL_IN_REG, 0, 2);
        b.add(LL_IN_LANE, 1, m_bits);
        b.add(LL_IN_LANE, 0, 6 - m_bits);
        b.add(LL_IN_REG, 0, 2 * m_bits - 8);
        return b.finish(out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_mfma_accumulator: out of host memory");
    }
}

ll_status ll_layout_mfma_operand(int m_bits, int k_reg_bits, ll_layout **out)
{
    try {
        if (ll_status st = check_out(out, 2); st != LL_OK) return st;
        if (m_bits != 4 && m_bits != 5) return fail(LL_ERR_INVALID_ARG, "operand tiles have 16 (m_bits 4) or 32 (m_bits 5) rows");
        if (k_reg_bits < 0 || k_reg_bits > 4) return fail(LL_ERR_INVALID_ARG, "k_reg_bits must be in [0, 4]");
        // a lane holds 2^k_reg_bits consecutive elements along K of one row; lanes run along the rows, then along K
        Builder b(2);
        b.add(LL_IN_REG, 1, k_reg_bits);
        b.add(LL_IN_LANE, 0, m_bits);
        b.add(LL_IN_LANE, 1, 6 - m_bits);
        return b.finish(out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_mfma_operand: out of host memory");
    }
}

ll_status ll_layout_mma_swizzle(int m_bits, int n_bits, int vec_elems, int per_phase, int max_phase, ll_layout **out)
{
    try {
        if (ll_status st = check_out(out, 2); st != LL_OK) return st;
        if (m_bits < 0 || n_bits < 0 || m_bits + n_bits < 1 || m_bits + n_bits > LL_MAX_BITS) return fail(LL_ERR_INVALID_ARG, "bad tensor size");
        if (!pow2(vec_elems) || !pow2(per_phase) || !pow2(max_phase)) return fail(LL_ERR_INVALID_ARG, "vec, per_phase and max_phase must be powers of two");
        if (log2i(vec_elems) + log2i(max_phase) > n_bits)
            return fail(LL_ERR_INVALID_ARG, "vec * max_phase exceeds the row length: the swizzle would leave the row");
        // [[I_n, C], [0, I_m]]: column bits keep their place; bit i of the row index also flips the
        // column bits c_i = (vec * ((2^i / per_phase) mod max_phase)) mod 2^n
        mat cols;
        for (int b = 0; b < n_bits; ++b) cols.push_back(vec(1) << b);
        for (int i = 0; i < m_bits; ++i) {
            const vec phase = ((vec(1) << i) / (vec)per_phase) % (vec)max_phase;
            const vec c = (phase * (vec)vec_elems) & ((vec(1) << n_bits) - 1);
            cols.push_back((vec(1) << (n_bits + i)) | c);
        }
        ll_in_dim in = {LL_IN_OFFSET, m_bits + n_bits};
        ll_out_dim o[2] = {{m_bits}, {n_bits}};
        return ll::make_layout(&in, 1, o, 2, cols, out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_mma_swizzle: out of host memory");
    }
}

ll_status ll_layout_classify(const ll_layout *layout, uint32_t *flags)
{
    try {
        if (!layout || !flags) return fail(LL_ERR_INVALID_ARG, "null argument");
        uint32_t f = 0;
        const int r = f2::rank(layout->bases);
        const bool surj = r == layout->d_out, inj = r == layout->d_in;
        if (surj) f |= LL_LAYOUT_SURJECTIVE;
        if (inj) f |= LL_LAYOUT_INJECTIVE;
        bool unit_or_zero = true, one_or_two = true;
        vec hit = 0;
        bool repeated = false;
        for (vec c : layout->bases) {
            const int pc = f2::popcount(c);
            unit_or_zero &= pc <= 1;
            one_or_two &= pc == 1 || pc == 2;
            if (pc == 1) {
                repeated |= (hit & c) != 0;
                hit |= c;
            }
        }
        bool hw_inputs = true;
        for (int i = 0; i < layout->n_in; ++i) hw_inputs &= layout->in_dims[i].label != LL_IN_OFFSET;
        if (surj && unit_or_zero && !repeated && hw_inputs) f |= LL_LAYOUT_DISTRIBUTED;
        if (surj && inj && one_or_two) f |= LL_LAYOUT_MEMORY;
        *flags = f;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_layout_classify: out of host memory");
    }
}

}  // extern "C"
