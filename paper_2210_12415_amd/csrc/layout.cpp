// Host-side layout algebra: parsing, primitive sequences (Table 1 of the
// paper), binding to a shape, offsets and their inverse.
#include <algorithm>
#include <cctype>

#include "common.h"
#include "layout_eval.h"

namespace alt {

namespace {

struct SymAtom {
    int dim;
    int64_t div;
    int64_t ext;
};

void clear_layout(alt_layout_t *l) { std::memset(l, 0, sizeof(*l)); }

}  // namespace

std::string layout_text(const alt_layout_t *l)
{
    char buf[256];
    std::string s;
    if (!l->separable) {
        s = "prims:";
        for (int q = 0; q < l->nprims; ++q) {
            const alt_prim_t &p = l->prims[q];
            std::snprintf(buf, sizeof buf, "%c%d(", p.kind == ALT_PRIM_SPLIT ? 's' : p.kind == ALT_PRIM_REORDER ? 'r' : 'f', p.dim);
            s += buf;
            int n = p.kind == ALT_PRIM_FUSE ? 0 : p.count;
            for (int j = 0; j < n; ++j) {
                std::snprintf(buf, sizeof buf, "%s%lld", j ? "," : "", (long long)p.v[j]);
                s += buf;
            }
            if (p.kind == ALT_PRIM_FUSE) { std::snprintf(buf, sizeof buf, "%d", p.count); s += buf; }
            s += ")";
        }
        return s;
    }
    for (int j = 0; j < l->nsub; ++j) {
        std::snprintf(buf, sizeof buf, "%sd%d/%lld", j ? "." : "", l->sub_dim[j], (long long)l->sub_div[j]);
        s += buf;
        if (l->sub_extent[j]) { std::snprintf(buf, sizeof buf, "x%lld", (long long)l->sub_extent[j]); s += buf; }
    }
    return s;
}

alt_status_t bind_layout(const alt_layout_t *l, int ndim, const int64_t *shape, BoundLayout *out,
                         std::string *err)
{
    auto bad = [&](alt_status_t s, const std::string &m) { if (err) *err = m; return s; };
    if (!l || !shape || !out) return bad(ALT_INVALID_ARG, "null layout or shape");
    if (ndim < 1 || ndim > ALT_MAX_RANK || l->ndim != ndim)
        return bad(ALT_SHAPE_MISMATCH, "layout rank does not match tensor rank");
    std::memset(out, 0, sizeof(*out));
    out->ndim = ndim;
    out->numel = 1;
    for (int d = 0; d < ndim; ++d) {
        if (shape[d] < 1) return bad(ALT_INVALID_ARG, "non-positive extent");
        out->shape[d] = shape[d];
        out->numel *= shape[d];
    }
    if (!l->separable) {
        if (l->nprims < 1 || l->nprims > ALT_MAX_PRIMS) return bad(ALT_INVALID_LAYOUT, "empty general layout");
        for (int d = 0; d < ndim; ++d)
            if (l->shape[d] != shape[d])
                return bad(ALT_SHAPE_MISMATCH, "primitive sequence was built for another shape");
        // A caller may have filled the descriptor by hand: walk the sequence with the same checks as
        // alt_layout_from_prims (dimension and count in range, split factors that multiply to the extent,
        // reorders that are permutations, fuses of adjacent dimensions), so that evaluating it never
        // indexes outside its arrays.
        std::vector<int64_t> cur(shape, shape + ndim);
        for (int q = 0; q < l->nprims; ++q) {
            const alt_prim_t &pr = l->prims[q];
            const int rank = (int)cur.size();
            std::vector<int64_t> ns;
            if (pr.kind == ALT_PRIM_SPLIT) {
                if (pr.dim < 0 || pr.dim >= rank || pr.count < 1 || pr.count > ALT_MAX_RANK || rank + pr.count - 1 > ALT_MAX_RANK)
                    return bad(ALT_INVALID_LAYOUT, "split outside the tensor's rank");
                int64_t prod = 1;
                for (int j = 0; j < pr.count; ++j) {
                    if (pr.v[j] < 1) return bad(ALT_INVALID_LAYOUT, "non-positive split factor");
                    prod *= pr.v[j];
                }
                if (prod != cur[pr.dim]) return bad(ALT_SHAPE_MISMATCH, "split factors do not multiply to the extent");
                for (int d = 0; d < rank; ++d) {
                    if (d != pr.dim) { ns.push_back(cur[d]); continue; }
                    for (int j = 0; j < pr.count; ++j) ns.push_back(pr.v[j]);
                }
            } else if (pr.kind == ALT_PRIM_REORDER) {
                if (pr.count != rank) return bad(ALT_INVALID_LAYOUT, "reorder of another rank");
                std::vector<int> seen(rank, 0);
                for (int j = 0; j < rank; ++j) {
                    const int64_t o = pr.v[j];
                    if (o < 0 || o >= rank || seen[o]) return bad(ALT_INVALID_LAYOUT, "reorder is not a permutation");
                    seen[o] = 1;
                    ns.push_back(cur[o]);
                }
            } else if (pr.kind == ALT_PRIM_FUSE) {
                if (pr.dim < 0 || pr.count < 1 || pr.dim + pr.count > rank) return bad(ALT_INVALID_LAYOUT, "fuse outside the tensor's rank");
                for (int d = 0; d < rank; ++d) {
                    if (d <= pr.dim || d >= pr.dim + pr.count) ns.push_back(cur[d]);
                    else ns.back() *= cur[d];
                }
            } else {
                return bad(ALT_INVALID_LAYOUT, "unknown primitive");
            }
            cur.swap(ns);
        }
        out->separable = 0;
        out->nprims = l->nprims;
        std::memcpy(out->prims, l->prims, sizeof(alt_prim_t) * l->nprims);
        return ALT_OK;
    }
    if (l->nsub < 1 || l->nsub > ALT_MAX_RANK) return bad(ALT_INVALID_LAYOUT, "bad piece count");
    out->separable = 1;
    out->nsub = l->nsub;
    for (int j = 0; j < l->nsub; ++j) {
        int d = l->sub_dim[j];
        if (d < 0 || d >= ndim || l->sub_div[j] < 1 || l->sub_extent[j] < 0)
            return bad(ALT_INVALID_LAYOUT, "bad piece");
        out->atom[j].dim = d;
        out->atom[j].group = l->sub_group[j];
        out->atom[j].div = l->sub_div[j];
        out->atom[j].ext = l->sub_extent[j];
    }
    // every logical dimension must be tiled exactly by its pieces
    for (int d = 0; d < ndim; ++d) {
        std::vector<int> ps;
        for (int j = 0; j < l->nsub; ++j)
            if (out->atom[j].dim == d) ps.push_back(j);
        if (ps.empty()) return bad(ALT_INVALID_LAYOUT, "a logical dimension has no piece");
        std::sort(ps.begin(), ps.end(), [&](int a, int b) { return out->atom[a].div < out->atom[b].div; });
        int64_t expect = 1;
        for (size_t t = 0; t < ps.size(); ++t) {
            Atom &a = out->atom[ps[t]];
            if (a.div != expect) return bad(ALT_INVALID_LAYOUT, "pieces of a dimension do not chain");
            bool top = t + 1 == ps.size();
            if (a.ext == 0) {
                if (!top) return bad(ALT_INVALID_LAYOUT, "only the outermost piece may be open");
                if (shape[d] % a.div != 0) {
                    char m[128];
                    std::snprintf(m, sizeof m, "block factor %lld does not divide extent %lld of dimension %d",
                                  (long long)a.div, (long long)shape[d], d);
                    return bad(ALT_SHAPE_MISMATCH, m);
                }
                a.ext = shape[d] / a.div;
            }
            expect = a.div * a.ext;
        }
        if (expect != shape[d]) {
            char m[128];
            std::snprintf(m, sizeof m, "pieces of dimension %d cover %lld, extent is %lld", d,
                          (long long)expect, (long long)shape[d]);
            return bad(ALT_SHAPE_MISMATCH, m);
        }
    }
    int64_t stride = 1;
    for (int j = l->nsub - 1; j >= 0; --j) {
        out->atom[j].stride = stride;
        stride *= out->atom[j].ext;
    }
    return ALT_OK;
}

bool layout_to_dim2(const BoundLayout &b, Dim2 *out)
{
    if (!b.separable) return false;
    for (int d = 0; d < b.ndim; ++d) {
        const Atom *inner = nullptr, *outer = nullptr;
        int n = 0;
        for (int j = 0; j < b.nsub; ++j) {
            const Atom &a = b.atom[j];
            if (a.dim != d || a.ext == 1) continue;
            ++n;
            if (a.div == 1) inner = &a; else outer = &a;
        }
        if (n > 2) return false;
        out[d].pad_ = 0;
        if (n == 0) { out[d].f = 1; out[d].so = 0; out[d].si = 0; out[d].fd = make_fastdiv(1); continue; }
        if (n == 1) {
            // the chain of divisors starts at 1, so a lone non-unit piece is the whole dimension
            const Atom *a = inner ? inner : outer;
            out[d].f = (int32_t)b.shape[d];
            out[d].so = 0;
            out[d].si = a->stride;
            out[d].fd = make_fastdiv((uint32_t)out[d].f);
            continue;
        }
        if (!inner || !outer || outer->div != inner->ext) return false;
        if (inner->ext > INT32_MAX) return false;
        out[d].f = (int32_t)inner->ext;
        out[d].si = inner->stride;
        out[d].so = outer->stride;
        out[d].fd = make_fastdiv((uint32_t)out[d].f);
    }
    return true;
}

}  // namespace alt

using namespace alt;

extern "C" {

alt_status_t alt_layout_parse(const char *text, alt_layout_t *out)
{
    if (!text || !out) return ALT_INVALID_ARG;
    clear_layout(out);
    const char *arrow = std::strstr(text, "->");
    if (!arrow) return ALT_INVALID_LAYOUT;
    std::string logical(text, arrow - text), physical(arrow + 2);
    int nd = (int)logical.size();
    if (nd < 1 || nd > ALT_MAX_RANK || physical.empty()) return ALT_INVALID_LAYOUT;
    for (int i = 0; i < nd; ++i) {
        if (!std::isupper((unsigned char)logical[i])) return ALT_INVALID_LAYOUT;
        for (int j = 0; j < i; ++j)
            if (logical[j] == logical[i]) return ALT_INVALID_LAYOUT;
    }
    struct Tok { int dim; int64_t factor; };       // factor 0 = the open (upper-case) piece
    std::vector<Tok> toks;
    size_t p = 0;
    while (p < physical.size()) {
        int64_t num = 0;
        bool has_num = false;
        while (p < physical.size() && std::isdigit((unsigned char)physical[p])) {
            num = num * 10 + (physical[p] - '0');
            has_num = true;
            if (num > (int64_t)1 << 40) return ALT_INVALID_LAYOUT;
            ++p;
        }
        if (p >= physical.size()) return ALT_INVALID_LAYOUT;
        char ch = physical[p++];
        if (!std::isalpha((unsigned char)ch)) return ALT_INVALID_LAYOUT;
        size_t pos = logical.find((char)std::toupper((unsigned char)ch));
        if (pos == std::string::npos) return ALT_INVALID_LAYOUT;
        if (std::isupper((unsigned char)ch)) {
            if (has_num) return ALT_INVALID_LAYOUT;
            toks.push_back({(int)pos, 0});
        } else {
            if (!has_num || num < 1) return ALT_INVALID_LAYOUT;
            toks.push_back({(int)pos, num});
        }
    }
    if ((int)toks.size() > ALT_MAX_RANK) return ALT_INVALID_LAYOUT;
    out->ndim = nd;
    out->nsub = (int)toks.size();
    out->separable = 1;
    for (int d = 0; d < nd; ++d) {
        int opens = 0;
        for (auto &t : toks) opens += (t.dim == d && t.factor == 0);
        if (opens != 1) return ALT_INVALID_LAYOUT;
    }
    for (size_t j = 0; j < toks.size(); ++j) {
        // significance: blocks written later are finer; the open piece is coarsest
        int64_t div = 1;
        if (toks[j].factor == 0) {
            for (auto &t : toks) if (t.dim == toks[j].dim && t.factor) div *= t.factor;
        } else {
            for (size_t t = j + 1; t < toks.size(); ++t)
                if (toks[t].dim == toks[j].dim && toks[t].factor) div *= toks[t].factor;
        }
        out->sub_dim[j] = toks[j].dim;
        out->sub_group[j] = (int)j;
        out->sub_div[j] = div;
        out->sub_extent[j] = toks[j].factor;
    }
    return ALT_OK;
}

alt_status_t alt_layout_from_prims(int ndim, const int64_t *shape, const alt_prim_t *seq, int nseq,
                                   alt_layout_t *out)
{
    if (!shape || !out || (nseq > 0 && !seq)) return ALT_INVALID_ARG;
    if (ndim < 1 || ndim > ALT_MAX_RANK || nseq < 0 || nseq > ALT_MAX_PRIMS) return ALT_INVALID_ARG;
    clear_layout(out);
    std::vector<std::vector<SymAtom>> dims(ndim);
    std::vector<int64_t> cur(ndim);
    for (int d = 0; d < ndim; ++d) {
        if (shape[d] < 1) return ALT_INVALID_ARG;
        dims[d] = {SymAtom{d, 1, shape[d]}};
        cur[d] = shape[d];
        out->shape[d] = shape[d];
    }
    bool separable = true;
    for (int q = 0; q < nseq; ++q) {
        const alt_prim_t &pr = seq[q];
        int rank = (int)cur.size();
        if (pr.kind == ALT_PRIM_SPLIT) {
            if (pr.dim < 0 || pr.dim >= rank || pr.count < 1 || pr.count > ALT_MAX_RANK) return ALT_INVALID_LAYOUT;
            if (rank + pr.count - 1 > ALT_MAX_RANK) return ALT_INVALID_LAYOUT;
            int64_t prod = 1;
            for (int j = 0; j < pr.count; ++j) {
                if (pr.v[j] < 1) return ALT_INVALID_LAYOUT;
                prod *= pr.v[j];
            }
            if (prod != cur[pr.dim]) return ALT_SHAPE_MISMATCH;
            // peel factors off the inner end of the piece list
            std::vector<SymAtom> rest = dims[pr.dim];
            std::vector<std::vector<SymAtom>> parts(pr.count);
            for (int j = pr.count - 1; j >= 0 && separable; --j) {
                int64_t need = pr.v[j];
                std::vector<SymAtom> got;
                while (need > 1) {
                    if (rest.empty()) { separable = false; break; }
                    SymAtom &a = rest.back();
                    if (a.ext == 1) { rest.pop_back(); continue; }
                    if (need % a.ext == 0) {
                        need /= a.ext;
                        got.insert(got.begin(), a);
                        rest.pop_back();
                    } else if (a.ext % need == 0) {
                        got.insert(got.begin(), SymAtom{a.dim, a.div, need});
                        a.div *= need;
                        a.ext /= need;
                        need = 1;
                    } else {
                        separable = false;
                        break;
                    }
                }
                if (got.empty()) got.push_back(SymAtom{rest.empty() ? dims[pr.dim][0].dim : rest.back().dim, 1, 1});
                parts[j] = got;
            }
            std::vector<std::vector<SymAtom>> nd;
            std::vector<int64_t> ns;
            for (int d = 0; d < rank; ++d) {
                if (d != pr.dim) { nd.push_back(dims[d]); ns.push_back(cur[d]); continue; }
                for (int j = 0; j < pr.count; ++j) { nd.push_back(parts[j]); ns.push_back(pr.v[j]); }
            }
            dims.swap(nd);
            cur.swap(ns);
        } else if (pr.kind == ALT_PRIM_REORDER) {
            if (pr.count != rank) return ALT_INVALID_LAYOUT;
            std::vector<int> seen(rank, 0);
            std::vector<std::vector<SymAtom>> nd(rank);
            std::vector<int64_t> ns(rank);
            for (int j = 0; j < rank; ++j) {
                int64_t o = pr.v[j];
                if (o < 0 || o >= rank || seen[o]) return ALT_INVALID_LAYOUT;
                seen[o] = 1;
                nd[j] = dims[o];
                ns[j] = cur[o];
            }
            dims.swap(nd);
            cur.swap(ns);
        } else if (pr.kind == ALT_PRIM_FUSE) {
            if (pr.dim < 0 || pr.count < 1 || pr.dim + pr.count > rank) return ALT_INVALID_LAYOUT;
            std::vector<std::vector<SymAtom>> nd;
            std::vector<int64_t> ns;
            for (int d = 0; d < rank; ++d) {
                if (d < pr.dim || d >= pr.dim + pr.count) { nd.push_back(dims[d]); ns.push_back(cur[d]); continue; }
                if (d == pr.dim) { nd.push_back({}); ns.push_back(1); }
                nd.back().insert(nd.back().end(), dims[d].begin(), dims[d].end());
                ns.back() *= cur[d];
            }
            dims.swap(nd);
            cur.swap(ns);
        } else {
            return ALT_INVALID_LAYOUT;
        }
    }
    out->ndim = ndim;
    out->nprims = nseq;
    for (int q = 0; q < nseq; ++q) out->prims[q] = seq[q];
    int total = 0;
    for (auto &g : dims) total += (int)g.size();
    if (separable && total <= ALT_MAX_RANK) {
        out->separable = 1;
        int j = 0;
        for (size_t g = 0; g < dims.size(); ++g)
            for (auto &a : dims[g]) {
                out->sub_dim[j] = a.dim;
                out->sub_group[j] = (int)g;
                out->sub_div[j] = a.div;
                out->sub_extent[j] = a.ext;
                ++j;
            }
        out->nsub = j;
        // the coarsest piece of each dimension is left open, as in parsed layouts
        for (int d = 0; d < ndim; ++d) {
            int top = -1;
            for (int t = 0; t < j; ++t)
                if (out->sub_dim[t] == d && (top < 0 || out->sub_div[t] > out->sub_div[top] ||
                                             (out->sub_div[t] == out->sub_div[top] && out->sub_extent[t] > 1)))
                    top = t;
            if (top >= 0 && out->sub_div[top] * out->sub_extent[top] == shape[d]) out->sub_extent[top] = 0;
        }
    } else {
        if (nseq == 0) return ALT_INVALID_LAYOUT;
        out->separable = 0;
    }
    return ALT_OK;
}

alt_status_t alt_layout_physical_shape(const alt_layout_t *l, const int64_t *shape, int64_t *out_shape,
                                       int *out_rank)
{
    if (!l || !shape || !out_shape || !out_rank) return ALT_INVALID_ARG;
    BoundLayout b;
    alt_status_t s = bind_layout(l, l->ndim, shape, &b, nullptr);
    if (s != ALT_OK) return s;
    if (b.separable) {
        int r = 0, last = -1;
        for (int j = 0; j < b.nsub; ++j) {
            if (j == 0 || b.atom[j].group != last) { out_shape[r++] = 1; last = b.atom[j].group; }
            out_shape[r - 1] *= b.atom[j].ext;
        }
        *out_rank = r;
        return ALT_OK;
    }
    std::vector<int64_t> cur(b.shape, b.shape + b.ndim);
    for (int q = 0; q < b.nprims; ++q) {
        const alt_prim_t &p = b.prims[q];
        std::vector<int64_t> ns;
        if (p.kind == ALT_PRIM_SPLIT) {
            for (int d = 0; d < (int)cur.size(); ++d) {
                if (d != p.dim) { ns.push_back(cur[d]); continue; }
                for (int j = 0; j < p.count; ++j) ns.push_back(p.v[j]);
            }
        } else if (p.kind == ALT_PRIM_REORDER) {
            for (int j = 0; j < p.count; ++j) ns.push_back(cur[p.v[j]]);
        } else {
            for (int d = 0; d < (int)cur.size(); ++d) {
                if (d <= p.dim || d >= p.dim + p.count) ns.push_back(cur[d]);
                else ns.back() *= cur[d];
            }
        }
        cur.swap(ns);
    }
    if ((int)cur.size() > ALT_MAX_RANK) return ALT_INVALID_LAYOUT;
    for (size_t d = 0; d < cur.size(); ++d) out_shape[d] = cur[d];
    *out_rank = (int)cur.size();
    return ALT_OK;
}

alt_status_t alt_layout_offset(const alt_layout_t *l, const int64_t *shape, const int64_t *idx,
                               int64_t *out_offset)
{
    if (!l || !shape || !idx || !out_offset) return ALT_INVALID_ARG;
    BoundLayout b;
    alt_status_t s = bind_layout(l, l->ndim, shape, &b, nullptr);
    if (s != ALT_OK) return s;
    for (int d = 0; d < b.ndim; ++d)
        if (idx[d] < 0 || idx[d] >= shape[d]) return ALT_INVALID_ARG;
    *out_offset = eval_offset(b, idx);
    return ALT_OK;
}

alt_status_t alt_layout_index_of(const alt_layout_t *l, const int64_t *shape, int64_t offset,
                                 int64_t *out_idx)
{
    if (!l || !shape || !out_idx) return ALT_INVALID_ARG;
    BoundLayout b;
    alt_status_t s = bind_layout(l, l->ndim, shape, &b, nullptr);
    if (s != ALT_OK) return s;
    if (offset < 0 || offset >= b.numel) return ALT_INVALID_ARG;
    for (int d = 0; d < b.ndim; ++d) out_idx[d] = 0;
    if (b.separable) {
        for (int j = 0; j < b.nsub; ++j) {
            const Atom &a = b.atom[j];
            out_idx[a.dim] += ((offset / a.stride) % a.ext) * a.div;
        }
        return ALT_OK;
    }
    // General form: record the shape before every primitive, decode the offset
    // under the final shape, then undo the primitives last to first.
    std::vector<std::vector<int64_t>> shapes;
    std::vector<int64_t> cur(b.shape, b.shape + b.ndim);
    for (int q = 0; q < b.nprims; ++q) {
        shapes.push_back(cur);
        const alt_prim_t &p = b.prims[q];
        std::vector<int64_t> ns;
        if (p.kind == ALT_PRIM_SPLIT) {
            for (int d = 0; d < (int)cur.size(); ++d) {
                if (d != p.dim) { ns.push_back(cur[d]); continue; }
                for (int j = 0; j < p.count; ++j) ns.push_back(p.v[j]);
            }
        } else if (p.kind == ALT_PRIM_REORDER) {
            for (int j = 0; j < p.count; ++j) ns.push_back(cur[p.v[j]]);
        } else {
            for (int d = 0; d < (int)cur.size(); ++d) {
                if (d <= p.dim || d >= p.dim + p.count) ns.push_back(cur[d]);
                else ns.back() *= cur[d];
            }
        }
        cur.swap(ns);
    }
    std::vector<int64_t> ix(cur.size());
    for (int d = (int)cur.size() - 1; d >= 0; --d) { ix[d] = offset % cur[d]; offset /= cur[d]; }
    for (int q = b.nprims - 1; q >= 0; --q) {
        const alt_prim_t &p = b.prims[q];
        const std::vector<int64_t> &before = shapes[q];
        std::vector<int64_t> prev(before.size());
        if (p.kind == ALT_PRIM_SPLIT) {
            int r = 0;
            for (int d = 0; d < (int)before.size(); ++d) {
                if (d != p.dim) { prev[d] = ix[r++]; continue; }
                int64_t v = 0;
                for (int j = 0; j < p.count; ++j) v = v * p.v[j] + ix[r++];
                prev[d] = v;
            }
        } else if (p.kind == ALT_PRIM_REORDER) {
            for (int j = 0; j < p.count; ++j) prev[p.v[j]] = ix[j];
        } else {
            int r = 0;
            for (int d = 0; d < (int)before.size();) {
                if (d != p.dim) { prev[d++] = ix[r++]; continue; }
                int64_t v = ix[r++];
                for (int t = p.dim + p.count - 1; t >= p.dim; --t) { prev[t] = v % before[t]; v /= before[t]; }
                d = p.dim + p.count;
            }
        }
        ix.swap(prev);
    }
    for (int d = 0; d < b.ndim; ++d) out_idx[d] = ix[d];
    return ALT_OK;
}

}  // extern "C"
