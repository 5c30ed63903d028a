// Label-wise product and left division of layouts, register permutation for vector tiles, and
// the contiguity utility (paper Def. "Product", Def. "Left Division", Sec. 5.3 "Using SIMD
// Hardware Primitives" / "Generalized Vectorization", Sec. 5.1 "Contiguous elements").
#include <algorithm>
#include <vector>

#include "layout.hpp"

using f2::mat;
using f2::vec;

namespace {

// position of bit 0 of logical dim j in the flattened index (last dim fastest)
int shift_of(const ll_out_dim *dims, int n, int j)
{
    int s = 0;
    for (int k = j + 1; k < n; ++k) s += dims[k].nbits;
    return s;
}

vec field(vec x, int shift, int bits) { return (x >> shift) & ((vec(1) << bits) - 1); }

// Re-pack a flattened value: field j of `x` (dims `from`) goes to dims `to` at bit `lift[j]` of field j.
vec repack(vec x, const ll_out_dim *from, const ll_out_dim *to, int n, const int *lift)
{
    vec r = 0;
    for (int j = 0; j < n; ++j)
        r |= field(x, shift_of(from, n, j), from[j].nbits) << (shift_of(to, n, j) + lift[j]);
    return r;
}

bool has_label(const ll_layout *l, int label)
{
    for (int i = 0; i < l->n_in; ++i)
        if (l->in_dims[i].label == label) return true;
    return false;
}

// Division proper on explicit columns (`cols` replaces layout->bases: the caller may have permuted them).
ll_status divide(const ll_layout *layout, const mat &cols, const ll_layout *tile, ll_layout **out)
{
    const int r = layout->n_out;
    ll_out_dim qdims[LL_MAX_OUT_DIMS];
    int zero[LL_MAX_OUT_DIMS] = {};
    vec tile_rows = 0;                               // rows of `layout` that belong to the tile
    for (int j = 0; j < r; ++j) {
        if (tile->out_dims[j].nbits > layout->out_dims[j].nbits)
            return ll::fail(LL_ERR_NOT_DIVISIBLE, "the tile is larger than the layout along logical dim %d", j);
        qdims[j].nbits = layout->out_dims[j].nbits - tile->out_dims[j].nbits;
        tile_rows |= ((vec(1) << tile->out_dims[j].nbits) - 1) << shift_of(layout->out_dims, r, j);
    }
    ll_in_dim qin[LL_MAX_IN_DIMS];
    mat qcols;
    for (int i = 0; i < layout->n_in; ++i) {
        const int label = layout->in_dims[i].label, n = layout->in_dims[i].nbits;
        const int nt = tile->bits_of(label);
        if (nt > n) return ll::fail(LL_ERR_NOT_DIVISIBLE, "the tile has %d bits of input label %d, the layout %d", nt, label, n);
        const int first = layout->first_bit_of(label), tfirst = tile->first_bit_of(label);
        for (int k = 0; k < nt; ++k) {
            // upper-left block: the tile itself, lower-left block: zero
            const vec want = repack(tile->bases[tfirst + k], tile->out_dims, layout->out_dims, r, zero);
            if (cols[first + k] != want)
                return ll::fail(LL_ERR_NOT_DIVISIBLE, "input bit %d of label %d does not map as the tile does", k, label);
        }
        for (int k = nt; k < n; ++k) {
            // upper-right block: zero
            if (cols[first + k] & tile_rows)
                return ll::fail(LL_ERR_NOT_DIVISIBLE, "input bit %d of label %d reaches into the tile's part of the tensor", k, label);
            vec q = 0;
            for (int j = 0; j < r; ++j)
                q |= field(cols[first + k], shift_of(layout->out_dims, r, j) + tile->out_dims[j].nbits, qdims[j].nbits)
                     << shift_of(qdims, r, j);
            qcols.push_back(q);
        }
        qin[i].label = label;
        qin[i].nbits = n - nt;
    }
    // affine layouts: the constant splits like a column does; its tile part must be the tile's own
    if ((layout->offset & tile_rows) != repack(tile->offset, tile->out_dims, layout->out_dims, r, zero))
        return ll::fail(LL_ERR_NOT_DIVISIBLE, "the constant of the layout does not contain the constant of the tile");
    vec qoff = 0;
    for (int j = 0; j < r; ++j)
        qoff |= field(layout->offset, shift_of(layout->out_dims, r, j) + tile->out_dims[j].nbits, qdims[j].nbits) << shift_of(qdims, r, j);
    const ll_status st = ll::make_layout(qin, layout->n_in, qdims, r, qcols, out);
    if (st == LL_OK) (*out)->offset = qoff;
    return st;
}

ll_status check_pair(const ll_layout *layout, const ll_layout *tile, ll_layout **out)
{
    if (!out) return ll::fail(LL_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!layout || !tile) return ll::fail(LL_ERR_INVALID_ARG, "null layout");
    if (layout->n_out != tile->n_out)
        return ll::fail(LL_ERR_DIM_MISMATCH, "layout and tile have %d and %d logical dims", layout->n_out, tile->n_out);
    for (int i = 0; i < tile->n_in; ++i)
        if (tile->in_dims[i].nbits > 0 && !has_label(layout, tile->in_dims[i].label))
            return ll::fail(LL_ERR_NOT_DIVISIBLE, "the layout has no input label %d", tile->in_dims[i].label);
    return LL_OK;
}

}  // namespace

extern "C" {

ll_status ll_product_dimwise(const ll_layout *a, const ll_layout *b, ll_layout **out)
{
    try {
        if (!out) return ll::fail(LL_ERR_INVALID_ARG, "out is null");
        *out = nullptr;
        if (!a || !b) return ll::fail(LL_ERR_INVALID_ARG, "null layout");
        if (a->n_out != b->n_out) return ll::fail(LL_ERR_DIM_MISMATCH, "factors have %d and %d logical dims", a->n_out, b->n_out);
        if (a->d_in + b->d_in > LL_MAX_BITS || a->d_out + b->d_out > LL_MAX_BITS)
            return ll::fail(LL_ERR_INVALID_ARG, "product exceeds %d bits", LL_MAX_BITS);
        const int r = a->n_out;
        ll_out_dim odims[LL_MAX_OUT_DIMS];
        int zero[LL_MAX_OUT_DIMS] = {}, above[LL_MAX_OUT_DIMS];
        for (int j = 0; j < r; ++j) {
            odims[j].nbits = a->out_dims[j].nbits + b->out_dims[j].nbits;
            above[j] = a->out_dims[j].nbits;                 // b's bits of a dim sit above a's
        }
        ll_in_dim dims[LL_MAX_IN_DIMS];
        int n = 0;
        bool has_offset = false, has_hw = false;
        mat cols;
        for (int label = LL_IN_REG; label <= LL_IN_OFFSET; ++label) {
            if (!has_label(a, label) && !has_label(b, label)) continue;
            (label == LL_IN_OFFSET ? has_offset : has_hw) = true;
            const int na = a->bits_of(label), nb = b->bits_of(label);
            dims[n].label = label;
            dims[n].nbits = na + nb;
            ++n;
            for (int k = 0; k < na; ++k) cols.push_back(repack(a->bases[a->first_bit_of(label) + k], a->out_dims, odims, r, zero));
            for (int k = 0; k < nb; ++k) cols.push_back(repack(b->bases[b->first_bit_of(label) + k], b->out_dims, odims, r, above));
        }
        if (has_offset && has_hw) return ll::fail(LL_ERR_DIM_MISMATCH, "cannot multiply a memory layout with a distributed layout");
        const ll_status st = ll::make_layout(dims, n, odims, r, cols, out);
        // affine factors: the constants combine dim by dim exactly as the images do
        if (st == LL_OK) (*out)->offset = repack(a->offset, a->out_dims, odims, r, zero) | repack(b->offset, b->out_dims, odims, r, above);
        return st;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_product_dimwise: out of host memory");
    }
}

ll_status ll_divide_left(const ll_layout *layout, const ll_layout *tile, ll_layout **out)
{
    try {
        if (ll_status st = check_pair(layout, tile, out); st != LL_OK) return st;
        return divide(layout, layout->bases, tile, out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_divide_left: out of host memory");
    }
}

ll_status ll_divide_left_permuted(const ll_layout *layout, const ll_layout *tile, int label, int32_t *perm, ll_layout **out)
{
    try {
        if (ll_status st = check_pair(layout, tile, out); st != LL_OK) return st;
        if (!perm) return ll::fail(LL_ERR_INVALID_ARG, "perm is null");
        const int n = layout->bits_of(label), nt = tile->bits_of(label);
        if (nt > n) return ll::fail(LL_ERR_NOT_DIVISIBLE, "the tile has %d bits of input label %d, the layout %d", nt, label, n);
        const int first = layout->first_bit_of(label), tfirst = tile->first_bit_of(label);
        int zero[LL_MAX_OUT_DIMS] = {};
        // The tile's columns are taken in order; each claims the first unused input bit of `label`
        // that maps as it does.  The unclaimed bits follow in their old order.
        std::vector<int> order;
        std::vector<bool> used((size_t)n, false);
        for (int k = 0; k < nt; ++k) {
            const vec want = repack(tile->bases[tfirst + k], tile->out_dims, layout->out_dims, layout->n_out, zero);
            int found = -1;
            for (int c = 0; c < n && found < 0; ++c)
                if (!used[(size_t)c] && layout->bases[first + c] == want) found = c;
            if (found < 0)
                return ll::fail(LL_ERR_NOT_DIVISIBLE, "no input bit of label %d maps as bit %d of the tile does", label, k);
            used[(size_t)found] = true;
            order.push_back(found);
        }
        for (int c = 0; c < n; ++c)
            if (!used[(size_t)c]) order.push_back(c);
        mat cols = layout->bases;
        for (int k = 0; k < n; ++k) {
            cols[first + k] = layout->bases[first + order[(size_t)k]];
            perm[k] = order[(size_t)k];
        }
        return divide(layout, cols, tile, out);
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_divide_left_permuted: out of host memory");
    }
}

ll_status ll_contiguity(const ll_layout *layout, int32_t *elems)
{
    try {
        if (!layout || !elems) return ll::fail(LL_ERR_INVALID_ARG, "null argument");
        *elems = 1;
        if (layout->n_in == 0 || layout->in_dims[0].label != LL_IN_REG) return LL_OK;
        // Logical elements 0..2^u-1 sit in registers 0..2^u-1 of one thread exactly when register bit
        // i maps to logical bit i for every i < u (the inverse is then the identity on that block).
        int u = 0;
        while (u < layout->in_dims[0].nbits && u < layout->d_out && layout->bases[(size_t)u] == (vec(1) << u)) ++u;
        // an affine constant with low bits set reverses or swaps elements inside such a block
        while (u > 0 && (layout->offset & ((vec(1) << u) - 1))) --u;
        *elems = 1 << u;
        return LL_OK;
    } catch (...) {   // nothing may propagate across the C ABI
        return ll::fail(LL_ERR_INVALID_ARG, "ll_contiguity: out of host memory");
    }
}

}  // extern "C"
