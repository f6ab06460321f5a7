// Perspectives as compile-time tokens.
//
// The paper's language gives every piece of device code a perspective: a level of the
// hierarchy (thread, block, grid) paired with a static count n, written level[n], which also
// says how the group is aligned -- a perspective of n units starts at a multiple of n
// (section 3.1).  A warp is thread[32] there; on gfx950 a wavefront is thread[64].  Code moves
// between perspectives with two constructs (section 3.2): `group`, which replicates a
// narrower perspective evenly over the current one, and `split`, which shards the current one
// into unequal branches that run side by side; both are legal only under divisibility and
// alignment conditions (typing rules T-Group and T-Split, section 4).  Every function
// declares the perspective it needs, and a call site must offer one that is at least as
// broad (section 3.5).  It is a type error to call an operation from a perspective that
// cannot perform it: a wave-collective matrix instruction from per-thread code, a block
// barrier from a single wave.  Perspectives are erased before code generation (section 5).
//
// Here a perspective is an empty token object whose type carries level and count:
//
//   persp::Threads<N>   thread[N]: N consecutive threads of a block, the first a multiple of N
//   persp::Blocks<N>    block[N]:  N consecutive workgroups of the grid, likewise aligned
//   persp::Block<T>     block[1] of a kernel launched with T threads per workgroup
//   persp::Grid         grid[1]
//
// with the usual names Lane = Threads<1>, Wave = Threads<64>, Workgroup = Block<256>.
// Holding a persp::Wave means "this code is executed by all 64 lanes of a wavefront,
// converged"; a function that needs that takes a persp::Wave parameter -- its `requires`
// bound.  A call site may pass any broader perspective of the same level whose count the
// required one divides (thread[256] where thread[64] is asked for: the function is then run by
// each of the four waves), and never a narrower or misaligned one: the conversion does not
// exist.  Tokens cannot be made from nothing: a kernel obtains the grid token at its entry and
// narrows it; there is no way back up.  The tokens are empty and every function that takes
// one is inlined, so they leave no trace in the machine code.
//
// What C++ cannot express and the paper's checker can: a token that is still in scope inside
// a divergent branch can be misused there (the rule for this code base: a branch on a per-lane
// condition only uses persp::Lane operations, and the branch that a split hands a token to is
// the only one that uses it); and nothing stops a device function other than a kernel from
// calling Grid::at_kernel_entry -- that call is reserved by convention to the first statement
// of a __global__ function, where the whole grid is present and converged.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

namespace prism {
namespace persp {

template <int N> class Threads;
template <int N> class Blocks;
template <int THREADS> class Block;
class Grid;

namespace detail {

// The condition of the typing rule for `split` (section 4, T-Split), for any number of
// branches: the branches fit side by side into the n units, every branch size divides n,
// and every branch starts at a multiple of its own size.  For two branches of sizes n1, n2 this
// is the paper's  n1 + n2 <= n,  n1 | n,  n2 | n,  n2 | n1 + n  (the second branch starts at n1).
template <int N, int OFFSET>
constexpr bool aligned_split() { return OFFSET <= N; }
template <int N, int OFFSET, int FIRST, int... REST>
constexpr bool aligned_split()
{
    return FIRST >= 1 && N % FIRST == 0 && OFFSET % FIRST == 0 && OFFSET + FIRST <= N &&
           aligned_split<N, OFFSET + FIRST, REST...>();
}

template <int I, int FIRST, int... REST>
struct nth { static constexpr int value = nth<I - 1, REST...>::value; static constexpr int offset = FIRST + nth<I - 1, REST...>::offset; };
template <int FIRST, int... REST>
struct nth<0, FIRST, REST...> { static constexpr int value = FIRST; static constexpr int offset = 0; };

}  // namespace detail

// The branches of a split of thread[N] into thread[N1], thread[N2], ...: branch I is run by the
// threads whose index inside the split perspective lies in [offset<I>, offset<I> + size<I>).
// All branches execute, side by side (unordered composition); threads beyond the last branch
// sit the split out.
template <int N, int... SIZES>
class Split {
    static_assert(sizeof...(SIZES) >= 1, "a split has at least one branch");
    static_assert(detail::aligned_split<N, 0, SIZES...>(),
                  "split: the branches must fit into the perspective side by side, every branch size must "
                  "divide its size, and every branch must start at a multiple of its own size (align to)");
    template <int> friend class Threads;
    __device__ constexpr Split() {}

public:
    template <int I> static constexpr int size() { return detail::nth<I, SIZES...>::value; }
    template <int I> static constexpr int offset() { return detail::nth<I, SIZES...>::offset; }
    // does the thread with this index inside the split perspective belong to branch I?
    template <int I> __device__ static constexpr bool holds(int index) { return index >= offset<I>() && index < offset<I>() + size<I>(); }
    template <int I> __device__ constexpr Threads<detail::nth<I, SIZES...>::value> branch() const;
};

// thread[N].
template <int N>
class Threads {
    static_assert(N >= 1, "a perspective holds at least one unit");
    template <int> friend class Threads;
    template <int> friend class Block;
    template <int, int...> friend class Split;
    __device__ constexpr Threads() {}

public:
    static constexpr int count = N;

    // `group` (T-Group): thread[M] replicated over this perspective; M must divide N.
    template <int M>
    __device__ constexpr Threads<M> group() const
    {
        static_assert(M >= 1 && N % M == 0, "group: a narrower perspective replicates evenly only when its size divides the current one");
        return Threads<M>();
    }
    // `split` (T-Split): unequal branches side by side, each aligned to its own size.
    template <int... SIZES>
    __device__ constexpr Split<N, SIZES...> split() const { return Split<N, SIZES...>(); }

    // A function that requires thread[M] may be called from any broader thread[N] (M divides
    // N): the call site's perspective converts; nothing converts the other way.
    template <int M, typename = typename std::enable_if<(M < N) && N % M == 0>::type>
    __device__ constexpr operator Threads<M>() const { return Threads<M>(); }

    // every thread of the perspective may run per-thread code
    __device__ constexpr Threads<1> lane() const { return Threads<1>(); }
};

template <int N, int... SIZES>
template <int I>
__device__ constexpr Threads<detail::nth<I, SIZES...>::value> Split<N, SIZES...>::branch() const
{
    return Threads<detail::nth<I, SIZES...>::value>();
}

using Lane = Threads<1>;
using Wave = Threads<64>;  // the wavefront of gfx950

// block[1] of a kernel whose workgroups have THREADS threads.
template <int THREADS>
class Block {
    static_assert(THREADS >= 64 && THREADS % 64 == 0, "workgroups are made of whole wavefronts");
    friend class Grid;
    template <int> friend class Blocks;
    __device__ constexpr Block() {}

public:
    static constexpr int threads = THREADS;
    // The block seen as its threads (the calculus's `destruct`, section 4): thread[THREADS].
    __device__ constexpr Threads<THREADS> destruct() const { return Threads<THREADS>(); }
    __device__ constexpr Wave wave() const { return Wave(); }
    // a function that requires thread[M] may be called at block level when M divides the block
    template <int M, typename = typename std::enable_if<THREADS % M == 0>::type>
    __device__ constexpr operator Threads<M>() const { return Threads<M>(); }
};

using Workgroup = Block<256>;  // every kernel of this library launches four wavefronts

// block[N]: N consecutive workgroups (the launch must supply a multiple of N of them).
template <int N>
class Blocks {
    static_assert(N >= 1, "a perspective holds at least one unit");
    friend class Grid;
    template <int> friend class Blocks;
    __device__ constexpr Blocks() {}

public:
    static constexpr int count = N;
    template <int M>
    __device__ constexpr Blocks<M> group() const
    {
        static_assert(M >= 1 && N % M == 0, "group: a narrower perspective replicates evenly only when its size divides the current one");
        return Blocks<M>();
    }
    template <int THREADS = 256>
    __device__ constexpr Block<THREADS> workgroup() const { return Block<THREADS>(); }
};

class Grid {
    __device__ constexpr Grid() {}

public:
    // Only the first statement of a __global__ function may call this: at kernel entry all
    // threads of the grid are present and converged.
    __device__ static constexpr Grid at_kernel_entry() { return Grid(); }
    // group(block[1]): the code that follows is written for one workgroup of THREADS threads
    template <int THREADS = 256>
    __device__ constexpr Block<THREADS> workgroup() const { return Block<THREADS>(); }
    // group(block[N]) for a grid launched with a multiple of N workgroups
    template <int N>
    __device__ constexpr Blocks<N> blocks() const { return Blocks<N>(); }
};

}  // namespace persp
}  // namespace prism
