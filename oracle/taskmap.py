"""Task mappings in pure Python, following Section 5.1 of the paper.  TEST INFRASTRUCTURE ONLY.

A task mapping assigns to each worker w in {0..n-1} an ordered list of tasks from the grid
{(t_0..t_{m-1}) : 0 <= t_i < d_i} (Section 5.1.1).  The two basic mappings and the composition
rule (Section 5.1.2) are written out below exactly as the definitions read.

Readings where the text is silent (its figures are not available):
  * tasks inside ``repeat`` run in row-major order (last index fastest);
  * ``spatial(d)`` gives worker w the w-th task in that same order;
  * in the composition's list comprehension the task of the first mapping is the outer
    variable -- the only order for which composition is associative as lists.
"""
from itertools import product


class TaskMapping:
    def __init__(self, num_workers, task_shape, fn):
        self.num_workers = int(num_workers)
        self.task_shape = tuple(int(d) for d in task_shape)
        self._fn = fn

    def __call__(self, w):
        if not 0 <= w < self.num_workers:
            raise IndexError("worker id out of range")
        return [tuple(t) for t in self._fn(w)]

    def __mul__(self, other):
        return compose(self, other)


def repeat(*d):
    """One worker executes the whole grid d, in row-major order."""
    tasks = list(product(*[range(x) for x in d]))
    return TaskMapping(1, d, lambda w: tasks)


def spatial(*d):
    """prod(d) workers, one task each: worker w owns the w-th grid point in row-major order."""
    n = 1
    for x in d:
        n *= x

    def fn(w):
        t = []
        for x in reversed(d):
            t.append(w % x)
            w //= x
        return [tuple(reversed(t))]

    return TaskMapping(n, d, fn)


def compose(f1, f2):
    """f3 = f1 o f2: n3 = n1*n2, d3 = d1 (.) d2, f3(w) = [t1 (.) d2 + t2 : t1 in f1(w // n2), t2 in f2(w % n2)]."""
    if len(f1.task_shape) != len(f2.task_shape):
        raise ValueError("task dimensions differ")
    n2, d2 = f2.num_workers, f2.task_shape
    shape = tuple(a * b for a, b in zip(f1.task_shape, d2))

    def fn(w):
        return [tuple(a * d + b for a, d, b in zip(t1, d2, t2)) for t1 in f1(w // n2) for t2 in f2(w % n2)]

    return TaskMapping(f1.num_workers * n2, shape, fn)
