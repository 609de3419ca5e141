// CPU oracle for layer-by-layer sparse-DNN inference.  TEST INFRASTRUCTURE ONLY:
// tests, the smoke check and the benchmark's cpu_baseline leg call it; the GPU
// library never does, and the two share no code.
//
// What it computes is the plain definition, iterated (Section II-A-1, Eq. 1,
// with the clipped ReLU defined next to it, and the outline in Alg. 1):
//
//     Y_{l+1}[r][j] = min(max( sum_k Y_l[r][idx_l[j][k]] * val_l[j][k] + bias[j], 0), 32)
//
// for all L layers l = 0..L-1, where idx_l[j][0..31] / val_l[j][0..31] are the 32
// stored connections of output neuron j (a row of the paper's W_l).  Feature
// rows are independent.  The only shortcut is the one the method itself takes
// (host loop of Listing 1): a row with no strictly positive output after a layer
// is dropped from the active list and never evaluated again; that is exact when
// every bias is <= 0, because a zero row then maps to a zero row.  A "no skip"
// mode evaluates every row at every layer so tests can confirm the equivalence.
//
// Readings where the paper is silent or inconsistent:
//  * result is Y_L (all L weight matrices applied), Alg. 1 says "Y_{L-1}";
//  * bias is one float per output neuron shared by all layers (Listings 1, 2);
//  * every output element is defined (non-positive -> 0), although the listings
//    only store positive ones;
//  * "active" means some clipped output is strictly > 0 (Listings 1, 2);
//  * accumulation: slot order k = 0..31, one fused multiply-add per connection
//    in the working precision, bias added last.
//
// General sparse layers (Section II-A-1: W_l may be any sparse matrix; Listing 1
// stores it in CSR): the *_csr entry points take, per layer, ptr[0..N] with the
// connections of output neuron j at positions ptr[j] .. ptr[j+1]-1 of idx / val, any
// number per neuron (none: the output is the clipped bias).  Same definition, same
// accumulation rule (stored order, one fused multiply-add each, bias last).
//
// Precision: float (the paper's FEATPREC) in spdnn_oracle_infer; double in
// spdnn_oracle_infer_f64 (used to bound the float rounding error in tests).
//
// Pins (tests/test_oracle_*.py): dense brute force on tiny N, layer-0 integer
// closed form, uniform-row closed form incl. the clip at 32, identity pattern,
// zero input, row independence, permutation equivariance, monotonicity,
// skip == no-skip, float vs double within the rounding bound; for the general
// (CSR) form: dense brute force with uneven neuron lengths, the constant-row closed
// form with per-neuron weight sums, neurons without connections, and invariance
// under appended zero-weight connections.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

template <typename T> inline T fma_t(T a, T b, T c);
template <> inline float fma_t<float>(float a, float b, float c) { return std::fmaf(a, b, c); }
template <> inline double fma_t<double>(double a, double b, double c) { return std::fma(a, b, c); }

constexpr int kNnz = 32;

// One feature row through one layer.  Returns the largest pre-clip value z.
// ptr == NULL: neuron j owns entries j*32 .. j*32+31; else entries ptr[j] .. ptr[j+1]-1.
template <typename T>
T layer_row(int32_t N, const int32_t* ptr, const int32_t* idx, const float* val, const float* bias,
            const T* in, T* out, bool* any_positive) {
    bool pos = false;
    T zmax = -INFINITY;
    for (int32_t j = 0; j < N; ++j) {
        T acc = 0;
        const size_t first = ptr ? (size_t)ptr[j] : (size_t)j * kNnz;
        const int cnt = ptr ? ptr[j + 1] - ptr[j] : kNnz;
        const int32_t* ij = idx + first;
        const float* vj = val + first;
        for (int k = 0; k < cnt; ++k) acc = fma_t<T>(in[ij[k]], (T)vj[k], acc);
        T z = acc + (T)bias[j];
        if (z > zmax) zmax = z;
        T y = (z < (T)0) ? (T)0 : (z > (T)32) ? (T)32 : z;
        out[j] = y;
        if (y > (T)0) pos = true;
    }
    *any_positive = pos;
    return zmax;
}

template <typename T>
int infer(int32_t N, int32_t L, const int32_t* const* ptr, const int32_t* const* idx, const float* const* val,
          const float* bias, const T* Y0, int32_t batch, int32_t no_skip,
          int32_t* n_active, int32_t* active_rows, T* Y_final,
          int32_t* active_per_layer, int32_t* fragile_layer, double fragile_eps,
          int32_t* layers_evaluated) {
    if (N < 1 || L < 0 || batch < 0 || !bias || (!Y0 && batch > 0) || !n_active) return -1;
    if (L > 0 && (!idx || !val)) return -1;
    const size_t n = (size_t)N;
    std::vector<T> cur((size_t)batch * n), nxt((size_t)batch * n);
    if (batch > 0) std::memcpy(cur.data(), Y0, sizeof(T) * (size_t)batch * n);
    // act[i] = original id of the i-th row still active (ascending).
    std::vector<int32_t> act(batch);
    for (int32_t r = 0; r < batch; ++r) act[r] = r;
    // alive[r] only matters in no-skip mode: rows stay in the loop but the
    // active list is still reported the same way.
    std::vector<char> alive(batch, 1);
    if (fragile_layer) for (int32_t r = 0; r < batch; ++r) fragile_layer[r] = -1;
    if (active_per_layer) active_per_layer[0] = batch;
    int32_t evaluated = 0;
    for (int32_t l = 0; l < L; ++l) {
        if (!no_skip && act.empty()) {           // nothing left: remaining layers keep it empty
            if (active_per_layer) active_per_layer[l + 1] = 0;
            continue;
        }
        if (!idx[l] || !val[l] || (ptr && !ptr[l])) return -2;  // layer needed but not provided
        ++evaluated;
        std::vector<int32_t> keep;
        const int32_t nrows = no_skip ? batch : (int32_t)act.size();
        for (int32_t i = 0; i < nrows; ++i) {
            const int32_t r = no_skip ? i : act[i];
            bool pos = false;
            T zmax = layer_row<T>(N, ptr ? ptr[l] : nullptr, idx[l], val[l], bias, &cur[(size_t)r * n], &nxt[(size_t)r * n], &pos);
            if (no_skip) {
                if (!alive[r]) continue;         // already dropped from the list
                if (!pos) alive[r] = 0;
            }
            if (fragile_layer && fragile_layer[r] < 0 && std::fabs((double)zmax) < fragile_eps)
                fragile_layer[r] = l;
            if (pos) keep.push_back(r);
        }
        act.swap(keep);
        cur.swap(nxt);
        if (active_per_layer) active_per_layer[l + 1] = (int32_t)act.size();
    }
    *n_active = (int32_t)act.size();
    for (size_t i = 0; i < act.size(); ++i) {
        if (active_rows) active_rows[i] = act[i];
        if (Y_final) std::memcpy(Y_final + i * n, &cur[(size_t)act[i] * n], sizeof(T) * n);
    }
    if (layers_evaluated) *layers_evaluated = evaluated;
    return 0;
}

}  // namespace

extern "C" {

// float path.  idx[l] / val[l]: N*32 entries, entry j*32+k = k-th connection of
// output neuron j; a NULL layer pointer is allowed only if no active row reaches
// that layer (returns -2 otherwise).  Y0: batch*N row-major.  Outputs: n_active,
// active_rows[0..n_active) ascending original row ids, Y_final[i*N..] = row
// active_rows[i] of Y_L (may be NULL), active_per_layer[0..L] (may be NULL; entry
// l = rows active on entry to layer l), fragile_layer[r] = first layer at which
// row r, while active, had |max_j z| < fragile_eps, else -1 (may be NULL),
// layers_evaluated = number of layers that had any row to evaluate (may be NULL).
// Returns 0, -1 on bad arguments, -2 on a missing layer.
int spdnn_oracle_infer(int32_t N, int32_t L, const int32_t* const* idx, const float* const* val,
                       const float* bias, const float* Y0, int32_t batch, int32_t no_skip,
                       int32_t* n_active, int32_t* active_rows, float* Y_final,
                       int32_t* active_per_layer, int32_t* fragile_layer, double fragile_eps,
                       int32_t* layers_evaluated) {
    return infer<float>(N, L, nullptr, idx, val, bias, Y0, batch, no_skip, n_active, active_rows, Y_final,
                        active_per_layer, fragile_layer, fragile_eps, layers_evaluated);
}

// Same in double precision (feature maps and accumulation in double).
int spdnn_oracle_infer_f64(int32_t N, int32_t L, const int32_t* const* idx, const float* const* val,
                           const float* bias, const double* Y0, int32_t batch, int32_t no_skip,
                           int32_t* n_active, int32_t* active_rows, double* Y_final,
                           int32_t* active_per_layer, int32_t* fragile_layer, double fragile_eps,
                           int32_t* layers_evaluated) {
    return infer<double>(N, L, nullptr, idx, val, bias, Y0, batch, no_skip, n_active, active_rows, Y_final,
                         active_per_layer, fragile_layer, fragile_eps, layers_evaluated);
}

// General sparse layers: ptr[l] has N+1 non-decreasing entries starting at 0; idx[l] /
// val[l] have ptr[l][N] entries.  Everything else as above.
int spdnn_oracle_infer_csr(int32_t N, int32_t L, const int32_t* const* ptr, const int32_t* const* idx,
                           const float* const* val, const float* bias, const float* Y0, int32_t batch,
                           int32_t no_skip, int32_t* n_active, int32_t* active_rows, float* Y_final,
                           int32_t* active_per_layer, int32_t* fragile_layer, double fragile_eps,
                           int32_t* layers_evaluated) {
    if (L > 0 && !ptr) return -1;
    return infer<float>(N, L, ptr, idx, val, bias, Y0, batch, no_skip, n_active, active_rows, Y_final,
                        active_per_layer, fragile_layer, fragile_eps, layers_evaluated);
}

int spdnn_oracle_infer_csr_f64(int32_t N, int32_t L, const int32_t* const* ptr, const int32_t* const* idx,
                               const float* const* val, const float* bias, const double* Y0, int32_t batch,
                               int32_t no_skip, int32_t* n_active, int32_t* active_rows, double* Y_final,
                               int32_t* active_per_layer, int32_t* fragile_layer, double fragile_eps,
                               int32_t* layers_evaluated) {
    if (L > 0 && !ptr) return -1;
    return infer<double>(N, L, ptr, idx, val, bias, Y0, batch, no_skip, n_active, active_rows, Y_final,
                         active_per_layer, fragile_layer, fragile_eps, layers_evaluated);
}

}  // extern "C"
