// Host-side linear algebra over F2 (paper Sec. 2.4, Sec. 4.2).
#include "f2.hpp"

namespace f2 {

mat compose(const mat &outer, const mat &inner)
{
    mat r(inner.size());
    for (size_t j = 0; j < inner.size(); ++j) r[j] = apply(outer, inner[j]);
    return r;
}

mat identity(int d)
{
    mat r(d);
    for (int k = 0; k < d; ++k) r[k] = vec(1) << k;
    return r;
}

bool Basis::add(vec v, vec tag, vec *dep_tag)
{
    while (v) {
        int t = top_bit(v);
        if (!has_[t]) {
            has_[t] = true;
            v_[t] = v;
            tag_[t] = tag;
            ++dim_;
            return true;
        }
        v ^= v_[t];
        tag ^= tag_[t];
    }
    if (dep_tag) *dep_tag = tag;
    return false;
}

vec Basis::reduce(vec v, vec *tag_out) const
{
    vec tag = 0;
    for (int t = 63; t >= 0 && v; --t) {
        if (((v >> t) & 1) && has_[t]) {
            v ^= v_[t];
            tag ^= tag_[t];
        }
    }
    if (tag_out) *tag_out = tag;
    return v;
}

mat Basis::vectors() const
{
    mat r;
    for (int t = 63; t >= 0; --t)
        if (has_[t]) r.push_back(v_[t]);
    return r;
}

int rank(const mat &vectors)
{
    Basis b;
    for (vec v : vectors) b.add(v);
    return b.dim();
}

bool right_inverse(const mat &m, int d_out, mat *inv)
{
    // Column k enters the basis tagged with the unit vector e_k of the INPUT space, so the tag of
    // a reduction is the combination of input columns that produces the reduced vector.
    Basis b;
    for (size_t k = 0; k < m.size(); ++k) b.add(m[k], vec(1) << k);
    if (b.dim() != d_out) return false;
    inv->assign(d_out, 0);
    for (int i = 0; i < d_out; ++i) {
        vec tag = 0;
        vec rest = b.reduce(vec(1) << i, &tag);
        if (rest) return false;
        (*inv)[i] = tag;      // M * tag = e_i, only pivot columns are used
    }
    return true;
}

bool invert(const mat &m, int d, mat *inv)
{
    if ((int)m.size() != d) return false;
    for (vec c : m)
        if (d < 64 && (c >> d)) return false;
    return right_inverse(m, d, inv);
}

mat intersect(const mat &a, const mat &b, int d)
{
    // Zassenhaus: reduce the rows (a_i | a_i) and (b_j | 0); rows whose first block vanishes
    // carry a basis of the intersection in the second block.  The first block is kept in the
    // HIGH bits so that elimination clears it first.
    Basis z;
    mat out;
    auto push = [&](vec hi, vec lo) {
        vec row = (hi << d) | lo;
        // manual insertion so that the remainder can be inspected
        vec r = z.reduce(row);
        if (r == 0) return;
        z.add(r);
    };
    for (vec x : a) push(x, x);
    for (vec x : b) push(x, 0);
    for (vec row : z.vectors())
        if ((row >> d) == 0 && row != 0) out.push_back(row);
    return out;
}

mat extend(const mat &sub, const mat &candidates)
{
    Basis b;
    for (vec v : sub) b.add(v);
    mat out;
    for (vec c : candidates)
        if (b.add(c)) out.push_back(c);
    return out;
}

mat complement(const mat &sub, int d)
{
    return extend(sub, identity(d));
}

}  // namespace f2
