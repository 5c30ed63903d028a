// Host-side linear algebra over F2 (paper Sec. 2.4 and Sec. 4.2).
//
// A matrix is stored by columns: cols[k] is the image of input bit k, a bit vector packed in a
// 64-bit word (bit i = row i).  Subspaces are stored as lists of spanning vectors.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace f2 {

using vec = uint64_t;
using mat = std::vector<vec>;   // columns

inline int popcount(vec x) { return __builtin_popcountll(x); }
inline int top_bit(vec x) { return 63 - __builtin_clzll(x); }   // x != 0

// y = M x : XOR of the columns selected by the set bits of x (Sec. 4.1).
inline vec apply(const vec *cols, int ncols, vec x)
{
    vec y = 0;
    for (int k = 0; k < ncols; ++k)
        if ((x >> k) & 1) y ^= cols[k];
    return y;
}
inline vec apply(const mat &m, vec x) { return apply(m.data(), (int)m.size(), x); }

// Matrix product outer * inner over F2 (Def. "Composition"): column j of the product is
// outer applied to column j of inner.
mat compose(const mat &outer, const mat &inner);

mat identity(int d);

// Echelon basis of a subspace with the combination of inserted vectors that produced each
// basis vector (used for inverses and membership tests).
class Basis {
public:
    // Insert v; `tag` is an arbitrary bit vector that is XOR-accumulated alongside (for example
    // the unit vector naming the inserted column).  Returns true if v was independent of the
    // basis so far.  When it returns false, *dep_tag (if given) receives the accumulated tag of
    // the dependency (tag of v XOR tags of the basis vectors that cancel it).
    bool add(vec v, vec tag = 0, vec *dep_tag = nullptr);
    bool contains(vec v) const { return reduce(v) == 0; }
    // Reduce v against the basis; *tag_out accumulates the tags of the basis vectors used.
    vec reduce(vec v, vec *tag_out = nullptr) const;
    int dim() const { return dim_; }
    mat vectors() const;      // the reduced basis vectors, highest leading bit first
private:
    vec v_[64] = {};
    vec tag_[64] = {};
    bool has_[64] = {};
    int dim_ = 0;
};

int rank(const mat &vectors);

// Inverse of a square invertible d x d matrix; returns false if singular.
bool invert(const mat &m, int d, mat *inv);

// Right inverse X (d_in x d_out, returned by columns, d_out of them) of a surjective d_out x d_in
// matrix: M X = I (Def. "Right Inverse").  Pivot columns are the leftmost independent input
// columns; free variables are zero.  Returns false if M is not surjective.
bool right_inverse(const mat &m, int d_out, mat *inv);

// A basis of span(a) intersected with span(b) (Zassenhaus algorithm); vectors live in d <= 31 bits.
mat intersect(const mat &a, const mat &b, int d);

// Vectors picked from `candidates` (in order) that extend span(sub) to span(sub + candidates).
mat extend(const mat &sub, const mat &candidates);

// A basis of a complement of span(sub) inside F2^d, built from unit vectors in ascending order.
mat complement(const mat &sub, int d);

}  // namespace f2
