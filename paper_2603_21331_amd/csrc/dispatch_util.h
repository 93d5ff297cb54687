// Host-side selection of kernel instantiations, shared by the libraries' launch code: the
// kernels take their per-thread work (16-byte chunks per thread, threads per row, lanes per
// row and elements per lane) as template arguments, and these helpers turn the run-time
// numbers into those arguments in one place.  The callback is a generic lambda that receives
// the numbers as std::integral_constant values, e.g.
//
//   with_shape<256, 8>(threads, chunks, [&](auto g, auto c) {
//     launch_row<DT, decltype(c)::value, decltype(g)::value>(a);
//   });
//
// Each (threads, chunks) pair a call site allows is one kernel instantiation, so the bounds
// given there are also what the build compiles.
#pragma once

#include <cstdint>
#include <type_traits>
#include <utility>

#include "packed_rows.h"

namespace rms {
namespace host {

template <int V>
using Const = std::integral_constant<int, V>;

// f(Const<C>) for C == chunks if FIRST <= chunks <= LAST; false (and no call) otherwise.
template <int FIRST, int LAST, typename F>
inline bool with_chunks(int chunks, F&& f) {
  if (chunks == FIRST) {
    f(Const<FIRST>{});
    return true;
  }
  if constexpr (FIRST < LAST) return with_chunks<FIRST + 1, LAST>(chunks, std::forward<F>(f));
  else return false;
}

// f(Const<G>, Const<C>) if threads == G and 1 <= chunks <= MAX_CHUNKS; false otherwise.  Call
// sites chain the thread counts they are built for with ||.
template <int G, int MAX_CHUNKS, typename F>
inline bool with_shape(int threads, int chunks, F&& f) {
  if (threads != G) return false;
  return with_chunks<1, MAX_CHUNKS>(chunks, [&](auto c) { f(Const<G>{}, c); });
}

// Whole 16-byte pieces of a row of N elements of `elem` bytes: what a workgroup of the
// element-addressed row kernels must hold wherever the row starts (vec_io.h, RowCut).
inline int64_t whole_pieces(int64_t N, int64_t elem) { return N * elem / 16; }

// Lane group of the LDS-staged short-row kernels (packed_rows.h) for rows of N elements: the
// narrowest group (1, 2, 4 ... 64 lanes) that holds the row with kPackElems elements per
// lane, and the elements per lane that the row then needs, (E - 1) * L < N <= E * L: 9 to 16,
// except that groups of one lane also take rows of 1 to 8 elements and groups of 8 lanes are
// what short rows of a multiple of `bank_bytes` bytes are widened to (rows of such a length on
// one or two lanes each put the lane groups of a wavefront on a few LDS banks: 64-byte rows 34
// us on one or two lanes against 27 on eight).  Calls f(Const<L>, Const<E>); N must be at most
// 64 * kPackElems.
template <int L, int E, typename F>
inline void with_packed_elems(int64_t N, F&& f) {
  if ((N + L - 1) / L == E) f(Const<L>{}, Const<E>{});
  else if constexpr (E > ((L == 1 || L == 8) ? 1 : kPackElems / 2 + 1)) with_packed_elems<L, E - 1>(N, std::forward<F>(f));
}

template <typename F>
inline void with_packed_shape(int64_t N, int64_t elem, int64_t bank_bytes, F&& f) {
  int64_t lanes = (N + kPackElems - 1) / kPackElems;   // lanes the row needs
  if ((N * elem) % bank_bytes == 0 && lanes < 8) lanes = 8;
  if (lanes <= 1) with_packed_elems<1, kPackElems>(N, f);
  else if (lanes <= 2) with_packed_elems<2, kPackElems>(N, f);
  else if (lanes <= 4) with_packed_elems<4, kPackElems>(N, f);
  else if (lanes <= 8) with_packed_elems<8, kPackElems>(N, f);
  else if (lanes <= 16) with_packed_elems<16, kPackElems>(N, f);
  else if (lanes <= 32) with_packed_elems<32, kPackElems>(N, f);
  else with_packed_elems<64, kPackElems>(N, f);
}

}  // namespace host
}  // namespace rms
