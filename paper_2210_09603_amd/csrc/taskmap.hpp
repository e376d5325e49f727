// Task mappings as compile-time templates (Section 5.1 of the Hidet paper).
//
// A task mapping assigns to every worker w in {0..workers-1} an ordered list of `tasks` grid
// points of the task domain {(i, j) : 0 <= i < shape0, 0 <= j < shape1}.  The two basic
// mappings and the composition rule of Section 5.1.2 are expressed as types whose members are
// all constexpr, so a kernel that walks `Map::task(worker, q)` for q = 0..tasks-1 in an unrolled
// loop pays nothing for the abstraction: every index folds into immediate offsets.
//
//   Repeat<d0, d1>   one worker runs the whole d0 x d1 grid, row-major order
//   Spatial<d0, d1>  d0*d1 workers, worker w owns grid point (w / d1, w % d1)
//   Compose<F1, F2>  workers = n1*n2, shape = d1 (.) d2,
//                    F3(w) = [ t1 (.) d2 + t2 : t1 in F1(w / n2), t2 in F2(w % n2) ]  (t1 outer)
//
// Workers are whatever the caller says they are: lanes of a wavefront, wavefronts of a
// workgroup, or workgroups of the grid.
#pragma once

namespace hidet {
namespace tmap {

struct Task {
  int i;
  int j;
};

template <int D0, int D1>
struct Repeat {
  static constexpr int workers = 1;
  static constexpr int tasks = D0 * D1;
  static constexpr int shape0 = D0;
  static constexpr int shape1 = D1;
  __host__ __device__ static constexpr Task task(int /*w*/, int q) { return Task{q / D1, q % D1}; }
};

template <int D0, int D1>
struct Spatial {
  static constexpr int workers = D0 * D1;
  static constexpr int tasks = 1;
  static constexpr int shape0 = D0;
  static constexpr int shape1 = D1;
  __host__ __device__ static constexpr Task task(int w, int /*q*/) { return Task{w / D1, w % D1}; }
};

template <class F1, class F2>
struct Compose {
  static constexpr int workers = F1::workers * F2::workers;
  static constexpr int tasks = F1::tasks * F2::tasks;
  static constexpr int shape0 = F1::shape0 * F2::shape0;
  static constexpr int shape1 = F1::shape1 * F2::shape1;
  __host__ __device__ static constexpr Task task(int w, int q) {
    const Task t1 = F1::task(w / F2::workers, q / F2::tasks);
    const Task t2 = F2::task(w % F2::workers, q % F2::tasks);
    return Task{t1.i * F2::shape0 + t2.i, t1.j * F2::shape1 + t2.j};
  }
};

// Left-to-right chain: Chain<A, B, C> = (A o B) o C = A o (B o C) (composition is associative).
template <class F, class... Rest>
struct ChainImpl {
  using type = Compose<F, typename ChainImpl<Rest...>::type>;
};
template <class F>
struct ChainImpl<F> {
  using type = F;
};
template <class... Fs>
using Chain = typename ChainImpl<Fs...>::type;

// Run-time block-level mapping spatial(tiles_m, tiles_n) with a grouped traversal: consecutive
// workgroup ids walk down `group` tile rows before moving to the next tile column, so that the
// workgroups resident together reuse the same A and B panels (the "thread block swizzle" the
// paper lists among the optimisations a tensor program must be able to express, Section 3.1).
struct GroupedSpatial {
  int tiles_m;
  int tiles_n;
  int group;
  __host__ __device__ Task task(int w) const {
    const int per_panel = group * tiles_n;
    const int panel = w / per_panel;
    const int first = panel * group;
    const int rows = (tiles_m - first) < group ? (tiles_m - first) : group;
    const int within = w - panel * per_panel;
    return Task{first + within % rows, within / rows};
  }
};

}  // namespace tmap
}  // namespace hidet
