// Host-side construction of the 28 x 28 matrix of +-1 used as the non-power-of-two factor of the
// rotation (rot_size = 28 * 2^t).  The paper only says that a large non-power-of-two rotation is
// split in one Cooley-Tukey step (Sec. 5.2); the factor chosen here is the Paley type-I Hadamard
// matrix of order 28 = 27 + 1 over GF(27) = GF(3)[t]/(t^3 + 2t + 1), element a0 + a1 t + a2 t^2
// numbered a0 + 3 a1 + 9 a2.
#include "basq_internal.h"

#include <mutex>

namespace basq {

namespace {

struct Gf27 { int a0, a1, a2; };

Gf27 from_index(int e) { return {e % 3, (e / 3) % 3, e / 9}; }
int to_index(const Gf27& x) { return x.a0 + 3 * x.a1 + 9 * x.a2; }

Gf27 add(const Gf27& x, const Gf27& y) { return {(x.a0 + y.a0) % 3, (x.a1 + y.a1) % 3, (x.a2 + y.a2) % 3}; }
Gf27 neg(const Gf27& x) { return {(3 - x.a0) % 3, (3 - x.a1) % 3, (3 - x.a2) % 3}; }
Gf27 scale(const Gf27& x, int c) { return {(x.a0 * c) % 3, (x.a1 * c) % 3, (x.a2 * c) % 3}; }

// x * t, using t^3 = -2t - 1 = t + 2 (mod 3)
Gf27 times_t(const Gf27& x) { return {(2 * x.a2) % 3, (x.a0 + x.a2) % 3, x.a1}; }

Gf27 mul(const Gf27& x, const Gf27& y) {
    const Gf27 xt = times_t(x);
    const Gf27 xtt = times_t(xt);
    return add(add(scale(x, y.a0), scale(xt, y.a1)), scale(xtt, y.a2));
}

int8_t g_h28[28 * 28];
std::once_flag g_once;

void build_h28() {
    bool is_square[27] = {false};
    for (int e = 1; e < 27; ++e) {
        const Gf27 x = from_index(e);
        is_square[to_index(mul(x, x))] = true;
    }
    // H = I + S,  S = [[0, 1^T], [-1, Q]],  Q[a][b] = chi(a - b)
    for (int i = 0; i < 28; ++i) {
        for (int j = 0; j < 28; ++j) {
            int v;
            if (i == 0) v = 1;
            else if (j == 0) v = -1;
            else if (i == j) v = 1;
            else {
                const int d = to_index(add(from_index(i - 1), neg(from_index(j - 1))));
                v = is_square[d] ? 1 : -1;
            }
            g_h28[i * 28 + j] = (int8_t)v;
        }
    }
}

}  // namespace

const int8_t* hadamard28_host() {
    std::call_once(g_once, build_h28);
    return g_h28;
}

}  // namespace basq
