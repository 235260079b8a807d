"""A small front-end for the core TC language -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

It reads the text of a tensor-comprehension function (appendix, "EBNF syntax for core TC"), infers the ranges of
the index variables in rounds (Section 3.1, "Range Inference") and evaluates the statements as float64 loop nests
(Section 3: one parallel loop per left-hand-side index, one reduction loop per index that occurs on the right
only, the right-hand side read in full before the left-hand side is assigned).  The tests use it to evaluate the
comprehensions of the GPU library from their text, as a second, independent route to the values that the
hand-written loop nests of tc_oracle.c produce, and to derive output extents instead of writing them down.

Nothing here is shared with the HIP path or with tc_oracle.c.  Plain numpy: the iteration space of a statement is
evaluated as one broadcast array expression (in slabs along the first parallel index when it is large), which is
the loop nest with its loops in an order that the semantics leave free.

What is covered: `def` with typed tensor and scalar arguments, `=` and the reductions `+=`, `*=`, `min=`, `max=`
with and without `!`, `where v in lo:hi`, numbers, unary minus and `!`, `+ - * / %`, comparisons, `&&`, `||`,
`c ? a : b`, `T.n` (extent of dimension n), tensor accesses with affine or data-dependent subscripts, and the
builtins listed in _BUILTINS.  Not covered: calls of one TC function from another (the paper marks them as
pseudo-code), recurrent definitions.

Readings where the paper leaves room (each is also listed in the design notes):
 * ranges are inferred per statement; an access to a tensor whose shape is already known -- an argument, or a
   tensor defined by another statement of the function -- constrains its subscripts, the left-hand side included.
   Shapes are settled in a first pass over the statements that repeats until nothing changes, so a statement such
   as `out(i,j) = bias(j)`, whose `i` no input constrains, takes the range of `i` from the shape that the
   accumulating statement after it gives to `out`;
 * a variable's range always starts at 0 unless a `where` clause says otherwise; if 0 is not admissible for some
   access the function is rejected;
 * `=` with an index that occurs on the right only is rejected (a reduction needs its operator);
 * a left-hand-side tensor may occur on the right only with exactly the subscripts of the left (the paper's
   syntactic check for in-place updates); an index may occur only once on the left.
"""
from __future__ import annotations

import math
import re
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


class TcError(ValueError):
    """Syntax error, failed range inference, or a rejected statement."""


# ------------------------------------------------------------------------------------------------ syntax tree
@dataclass
class Num:
    value: object  # int or float


@dataclass
class Name:
    id: str


@dataclass
class Unary:
    op: str
    a: object


@dataclass
class Binary:
    op: str
    a: object
    b: object


@dataclass
class Ternary:
    c: object
    a: object
    b: object


@dataclass
class Extent:
    tensor: str
    dim: int


@dataclass
class Call:
    name: str
    args: list


@dataclass
class Arg:
    name: str
    scalar_type: str
    shape: Optional[List[str]]  # None for a scalar argument; entries are size symbols or decimal numbers


@dataclass
class Stmt:
    lhs: str
    lhs_idx: List[str]
    op: str  # '=', '+=', '*=', 'min=', 'max=' with an optional trailing '!'
    rhs: object
    where: Dict[str, Tuple[object, object]] = field(default_factory=dict)


@dataclass
class Func:
    name: str
    args: List[Arg]
    returns: List[str]
    stmts: List[Stmt]


# ------------------------------------------------------------------------------------------------ lexer, parser
_WS = re.compile(r"(\s+|#[^\n]*)+")
_NUMBER = re.compile(r"""(
    0[xX][0-9a-fA-F]+[uUlL]*
  | (\d+\.\d*|\.\d+)([eE][+-]?\d+)?[fFlL]?
  | \d+[eE][+-]?\d+[fFlL]?
  | \d+[uUlL]*
  )(?![_a-zA-Z0-9])""", re.X)
_IDENT = re.compile(r"[_a-zA-Z0-9]*[_a-zA-Z][_a-zA-Z0-9]*")  # may start with digits as long as it holds a letter (2LUT)
_EXTENT = re.compile(r"\.(\d+)(?![_a-zA-Z0-9.])")             # T.0 directly after an identifier
_OP = re.compile(r"\+=!|\*=!|\+=|\*=|->|==|!=|<=|>=|&&|\|\||[-+*/%<>!?:=(),{}]")
_INT_TYPES = ("int", "int32", "int64", "uint32", "uint8", "byte", "long", "bool")
_FLOAT_TYPES = ("float", "double", "half")


def _lex(text: str):
    out, pos = [], 0
    while pos < len(text):
        m = _WS.match(text, pos)
        if m:
            pos = m.end()
            continue
        m = _NUMBER.match(text, pos)  # C number syntax wins over an identifier that starts with digits
        if m:
            tok = m.group()
            if tok.lower().startswith("0x"):
                out.append(("num", int(tok.rstrip("uUlL"), 16)))
            elif re.fullmatch(r"\d+[uUlL]*", tok):
                out.append(("num", int(tok.rstrip("uUlL"))))
            else:
                out.append(("num", float(tok.rstrip("fFlL"))))
            pos = m.end()
            continue
        m = _IDENT.match(text, pos)
        if m:
            out.append(("id", m.group()))
            pos = m.end()
            e = _EXTENT.match(text, pos)
            if e:
                out += [("op", "."), ("num", int(e.group(1)))]
                pos = e.end()
            continue
        m = _OP.match(text, pos)
        if not m:
            raise TcError("unexpected character %r at offset %d" % (text[pos], pos))
        out.append(("op", m.group()))
        pos = m.end()
    out.append(("end", None))
    return out


class _Parser:
    def __init__(self, text):
        self.t = _lex(text)
        self.i = 0

    def peek(self, k=0):
        return self.t[min(self.i + k, len(self.t) - 1)]

    def take(self):
        tok = self.t[self.i]
        self.i += 1
        return tok

    def at(self, kind, val=None, k=0):
        tk = self.peek(k)
        return tk[0] == kind and (val is None or tk[1] == val)

    def expect(self, kind, val=None):
        tk = self.take()
        if tk[0] != kind or (val is not None and tk[1] != val):
            raise TcError("expected %s, found %r" % (val or kind, tk[1]))
        return tk[1]

    # func ::= 'def' id '(' arg_list ')' '->' '(' return_list ')' '{' stmt_list '}'
    def func(self) -> Func:
        if self.expect("id") != "def":
            raise TcError("a TC function starts with 'def'")
        name = self.expect("id")
        self.expect("op", "(")
        args = []
        while not self.at("op", ")"):
            args.append(self.arg())
            if not self.at("op", ")"):
                self.expect("op", ",")
        self.expect("op", ")")
        self.expect("op", "->")
        self.expect("op", "(")
        rets = [self.expect("id")]
        while self.at("op", ","):
            self.take()
            rets.append(self.expect("id"))
        self.expect("op", ")")
        self.expect("op", "{")
        stmts = []
        while not self.at("op", "}"):
            stmts.append(self.stmt())
        self.expect("op", "}")
        self.expect("end")
        return Func(name, args, rets, stmts)

    def arg(self) -> Arg:
        st = self.expect("id")
        if st not in _INT_TYPES + _FLOAT_TYPES:
            raise TcError("unknown scalar type %r" % st)
        shape = None
        if self.at("op", "("):
            self.take()
            shape = []
            while not self.at("op", ")"):
                tk = self.take()
                if tk[0] not in ("id", "num"):
                    raise TcError("a shape lists size names or numbers")
                shape.append(str(tk[1]))
                if not self.at("op", ")"):
                    self.expect("op", ",")
            self.take()
        return Arg(self.expect("id"), st, shape)

    # stmt ::= id '(' id_list ')' [ '=' | reduction ] exp [ 'where' range_constraint_list ]
    def stmt(self) -> Stmt:
        lhs = self.expect("id")
        self.expect("op", "(")
        idx = []
        while not self.at("op", ")"):
            idx.append(self.expect("id"))
            if not self.at("op", ")"):
                self.expect("op", ",")
        self.take()
        if self.at("id") and self.peek()[1] in ("min", "max") and self.at("op", "=", 1):
            op = self.take()[1] + self.take()[1]
            if self.at("op", "!"):
                self.take()
                op += "!"
        else:
            op = self.expect("op")
            if op not in ("=", "+=", "*=", "+=!", "*=!"):
                raise TcError("expected '=' or a reduction operator, found %r" % op)
        rhs = self.exp()
        where = {}
        if self.at("id", "where"):
            self.take()
            while True:
                v = self.expect("id")
                if self.expect("id") != "in":
                    raise TcError("a range constraint reads 'v in lo:hi'")
                lo = self.exp(no_ternary=True)
                self.expect("op", ":")
                hi = self.exp(no_ternary=True)
                where[v] = (lo, hi)
                if not self.at("op", ","):
                    break
                self.take()
        return Stmt(lhs, idx, op, rhs, where)

    # precedence, lowest first: ?:  ||  &&  comparisons  + -  * / %  unary  primary
    def exp(self, no_ternary=False):
        c = self.binary(0)
        if not no_ternary and self.at("op", "?"):
            self.take()
            a = self.exp()
            self.expect("op", ":")
            return Ternary(c, a, self.exp())
        return c

    _LEVELS = [("||",), ("&&",), ("==", "!=", "<", "<=", ">", ">="), ("+", "-"), ("*", "/", "%")]

    def binary(self, level):
        if level == len(self._LEVELS):
            return self.unary()
        a = self.binary(level + 1)
        while self.at("op") and self.peek()[1] in self._LEVELS[level]:
            op = self.take()[1]
            a = Binary(op, a, self.binary(level + 1))
        return a

    def unary(self):
        if self.at("op", "-") or self.at("op", "!"):
            return Unary(self.take()[1], self.unary())
        return self.primary()

    def primary(self):
        tk = self.take()
        if tk[0] == "num":
            return Num(tk[1])
        if tk[0] == "op" and tk[1] == "(":
            e = self.exp()
            self.expect("op", ")")
            return e
        if tk[0] != "id":
            raise TcError("unexpected %r in an expression" % (tk[1],))
        if self.at("op", "."):
            self.take()
            return Extent(tk[1], int(self.expect("num")))
        if self.at("op", "("):
            self.take()
            args = []
            while not self.at("op", ")"):
                args.append(self.exp())
                if not self.at("op", ")"):
                    self.expect("op", ",")
            self.take()
            return Call(tk[1], args)
        return Name(tk[1])


def parse(text: str) -> Func:
    """Parse the text of one TC function."""
    return _Parser(text).func()


# ------------------------------------------------------------------------------------------------ range inference
_BUILTINS = {
    "fmaxf": np.maximum, "fmax": np.maximum, "max": np.maximum, "fminf": np.minimum, "fmin": np.minimum,
    "min": np.minimum, "exp": np.exp, "expf": np.exp, "log": np.log, "logf": np.log, "sqrt": np.sqrt,
    "sqrtf": np.sqrt, "tanh": np.tanh, "tanhf": np.tanh, "fabs": np.abs, "fabsf": np.abs, "abs": np.abs,
    "pow": np.power, "powf": np.power,
}


def _walk(e):
    """All nodes of an expression."""
    yield e
    if isinstance(e, Unary):
        yield from _walk(e.a)
    elif isinstance(e, Binary):
        yield from _walk(e.a)
        yield from _walk(e.b)
    elif isinstance(e, Ternary):
        for s in (e.c, e.a, e.b):
            yield from _walk(s)
    elif isinstance(e, Call):
        for s in e.args:
            yield from _walk(s)


def _affine(e, consts, is_index):
    """e as {index variable: integer coefficient, None: integer constant}, or None if e is not an affine
    integer function of the index variables (consts: names with known integer values)."""
    if isinstance(e, Num):
        return {None: e.value} if isinstance(e.value, int) else None
    if isinstance(e, Name):
        if e.id in consts:
            return {None: consts[e.id]} if isinstance(consts[e.id], int) else None
        return {e.id: 1, None: 0} if is_index(e.id) else None
    if isinstance(e, Unary) and e.op == "-":
        a = _affine(e.a, consts, is_index)
        return None if a is None else {k: -v for k, v in a.items()}
    if isinstance(e, Binary) and e.op in ("+", "-", "*"):
        a, b = _affine(e.a, consts, is_index), _affine(e.b, consts, is_index)
        if a is None or b is None:
            return None
        if e.op == "*":
            if len(a) > 1 and len(b) > 1:
                return None  # a product of two index expressions
            if len(a) > 1:
                a, b = b, a
            c = a.get(None, 0)
            return {k: c * v for k, v in b.items()}
        sgn = 1 if e.op == "+" else -1
        out = dict(a)
        for k, v in b.items():
            out[k] = out.get(k, 0) + sgn * v
        return out
    return None


def _accesses(e, tensors):
    """(tensor name, subscript list) of every tensor access inside e, nested ones included."""
    for n in _walk(e):
        if isinstance(n, Call) and n.name in tensors:
            yield n.name, n.args


def _index_vars(stmt: Stmt, known_names) -> List[str]:
    seen = []
    for v in stmt.lhs_idx:
        if v in known_names:
            raise TcError("left-hand-side index %r is the name of an argument or size" % v)
        if v not in seen:
            seen.append(v)
    for n in _walk(stmt.rhs):
        if isinstance(n, Name) and n.id not in known_names and n.id not in seen:
            seen.append(n.id)
    return seen


def _infer_stmt(stmt: Stmt, shapes: Dict[str, Tuple[int, ...]], consts: Dict[str, object]):
    """Ranges {index variable: (lo, hi)} of one statement, or None if a tensor it reads or writes has no shape
    yet and the ranges cannot be settled without it.  Raises TcError when inference fails for good."""
    for n in _walk(stmt.rhs):
        if isinstance(n, Name) and n.id not in consts and (n.id in shapes or n.id == stmt.lhs):
            raise TcError("tensor %s is used without subscripts" % n.id)
    ivars = _index_vars(stmt, set(consts))
    is_index = lambda name: name in ivars  # noqa: E731
    ranges: Dict[str, Tuple[int, int]] = {}
    for v, (lo, hi) in stmt.where.items():
        a, b = _affine(lo, consts, lambda n: False), _affine(hi, consts, lambda n: False)
        if a is None or b is None:
            raise TcError("the bounds of 'where %s in lo:hi' must be integer constants" % v)
        ranges[v] = (a[None], b[None])
    unresolved = [v for v in ivars if v not in ranges]

    # every affine subscript of every access to a tensor of known shape is one constraint: 0 <= e < extent
    cons = []
    acc = list(_accesses(stmt.rhs, shapes))
    missing_shape = any(isinstance(n, Call) and n.name not in shapes and n.name not in _BUILTINS
                        for n in _walk(stmt.rhs))
    if stmt.lhs in shapes:
        acc.append((stmt.lhs, [Name(v) for v in stmt.lhs_idx]))
    for name, subs in acc:
        if len(subs) != len(shapes[name]):
            raise TcError("%s has %d dimensions, accessed with %d subscripts" % (name, len(shapes[name]), len(subs)))
        for d, s in enumerate(subs):
            aff = _affine(s, consts, is_index)
            if aff is not None:
                cons.append((aff, shapes[name][d]))

    while unresolved:
        found: Dict[str, Tuple[int, int]] = {}
        for aff, extent in cons:
            open_vars = [v for v in aff if v is not None and aff[v] != 0 and v in unresolved]
            if len(open_vars) != 1:
                continue
            v = open_vars[0]
            a = aff[v]
            # the rest of the expression over the ranges already resolved: [rmin, rmax]
            rmin = rmax = aff.get(None, 0)
            for u, c in aff.items():
                if u is None or u == v or c == 0:
                    continue
                lo, hi = ranges[u]
                if hi <= lo:
                    continue
                ends = (c * lo, c * (hi - 1))
                rmin += min(ends)
                rmax += max(ends)
            # for all values of the rest: 0 <= a v + rest <= extent - 1
            if a > 0:
                vlo, vhi = math.ceil(-rmin / a), math.floor((extent - 1 - rmax) / a)
            else:
                vlo, vhi = math.ceil((extent - 1 - rmax) / a), math.floor(-rmin / a)
            if v in found:
                vlo, vhi = max(vlo, found[v][0]), min(vhi, found[v][1])
            found[v] = (vlo, vhi)
        if not found:
            if missing_shape or stmt.lhs not in shapes:
                return None  # perhaps another statement settles the shape of a tensor used here
            raise TcError("cannot infer the range of %s: add a where clause" % ", ".join(unresolved))
        for v, (vlo, vhi) in found.items():
            if vlo > 0:
                raise TcError("index %s cannot start at 0 here: add a where clause" % v)
            ranges[v] = (0, max(vhi + 1, 0))
            unresolved.remove(v)
    if missing_shape:
        return None
    return {v: ranges[v] for v in ivars}


@dataclass
class Plan:
    """What inference settles for a call: sizes, tensor shapes and the ranges of every statement."""
    sizes: Dict[str, int]
    shapes: Dict[str, Tuple[int, ...]]
    ranges: List[Dict[str, Tuple[int, int]]]


def infer(func: Func, arg_shapes: Dict[str, Tuple[int, ...]], scalars: Optional[Dict[str, object]] = None) -> Plan:
    """Bind the size symbols to the extents of the actual arguments and infer all ranges and output shapes."""
    scalars = dict(scalars or {})
    sizes: Dict[str, int] = {}
    shapes: Dict[str, Tuple[int, ...]] = {}
    consts: Dict[str, object] = {}
    for a in func.args:
        if a.shape is None:
            if a.name not in scalars:
                raise TcError("scalar argument %s has no value" % a.name)
            v = scalars[a.name]
            consts[a.name] = int(v) if a.scalar_type in _INT_TYPES else float(v)
            continue
        if a.name not in arg_shapes:
            raise TcError("tensor argument %s has no shape" % a.name)
        shp = tuple(int(x) for x in arg_shapes[a.name])
        if len(shp) != len(a.shape):
            raise TcError("%s is declared with %d dimensions, got %d" % (a.name, len(a.shape), len(shp)))
        for sym, ext in zip(a.shape, shp):
            if sym.isdigit():
                if int(sym) != ext:
                    raise TcError("%s: extent %d where %s is declared" % (a.name, ext, sym))
            elif sizes.setdefault(sym, ext) != ext:
                raise TcError("size %s is %d in one argument and %d in another" % (sym, sizes[sym], ext))
        shapes[a.name] = shp
    for s, v in sizes.items():
        if s in consts:
            raise TcError("%s names both a size and a scalar argument" % s)
        consts[s] = v  # a tensor may share its name with a size (listing sconv2d: W): accesses are calls, sizes are not

    inputs = set(shapes)
    ranges: List[Optional[dict]] = [None] * len(func.stmts)
    progress = True
    while progress and any(r is None for r in ranges):
        progress = False
        for i, st in enumerate(func.stmts):
            if ranges[i] is not None:
                continue
            if st.lhs in inputs:
                raise TcError("%s is an input; statements define outputs and temporaries" % st.lhs)
            _check_in_place(st)
            r = _infer_stmt(st, shapes, consts)
            if r is None:
                continue
            rhs_only = [v for v in r if v not in st.lhs_idx]
            if st.op == "=" and rhs_only:
                raise TcError("'=' with %s on the right only: a reduction needs its operator" % ", ".join(rhs_only))
            shape = tuple(r[v][1] for v in st.lhs_idx)
            if st.lhs in shapes:
                if any(h > e for h, e in zip(shape, shapes[st.lhs])):
                    raise TcError("statement %d writes outside %s" % (i, st.lhs))
            else:
                if any(r[v][0] != 0 for v in st.lhs_idx):
                    raise TcError("the first definition of %s must start every index at 0" % st.lhs)
                shapes[st.lhs] = shape
            ranges[i] = r
            progress = True
    if any(r is None for r in ranges):
        bad = [i for i, r in enumerate(ranges) if r is None]
        raise TcError("cannot infer the ranges of statement(s) %s: add where clauses" % bad)
    for name in func.returns:
        if name not in shapes or name in inputs:
            raise TcError("output %s is never defined" % name)
    return Plan(sizes, shapes, ranges)  # type: ignore[arg-type]


def _check_in_place(st: Stmt) -> None:
    if len(set(st.lhs_idx)) != len(st.lhs_idx):
        raise TcError("an index occurs twice on the left-hand side of %s" % st.lhs)
    for name, subs in _accesses(st.rhs, {st.lhs}):
        same = len(subs) == len(st.lhs_idx) and all(isinstance(s, Name) and s.id == v for s, v in zip(subs, st.lhs_idx))
        if not same:
            raise TcError("%s is read with subscripts other than those it is written with" % name)


# ------------------------------------------------------------------------------------------------ evaluation
_SLAB_ELEMS = 1 << 24  # iteration points evaluated at once


def _eval(e, env, tensors, consts):
    if isinstance(e, Num):
        return e.value
    if isinstance(e, Name):
        if e.id in env:
            return env[e.id]
        if e.id in consts:
            return consts[e.id]
        raise TcError("unknown name %s" % e.id)
    if isinstance(e, Extent):
        return tensors[e.tensor].shape[e.dim]
    if isinstance(e, Unary):
        a = _eval(e.a, env, tensors, consts)
        return -a if e.op == "-" else np.logical_not(a)
    if isinstance(e, Ternary):
        return np.where(_eval(e.c, env, tensors, consts), _eval(e.a, env, tensors, consts),
                        _eval(e.b, env, tensors, consts))
    if isinstance(e, Binary):
        a, b = _eval(e.a, env, tensors, consts), _eval(e.b, env, tensors, consts)
        ints = all(isinstance(x, (int, np.integer)) or (isinstance(x, np.ndarray) and x.dtype.kind in "iu") for x in (a, b))
        if e.op == "+":
            return a + b
        if e.op == "-":
            return a - b
        if e.op == "*":
            return a * b
        if e.op == "/":
            if ints:  # C semantics: truncation towards zero
                q = np.abs(a) // np.abs(b)
                return q * np.sign(a) * np.sign(b)
            return a / b
        if e.op == "%":
            return np.fmod(a, b)
        return {"==": np.equal, "!=": np.not_equal, "<": np.less, "<=": np.less_equal, ">": np.greater,
                ">=": np.greater_equal, "&&": np.logical_and, "||": np.logical_or}[e.op](a, b)
    if isinstance(e, Call):
        args = [_eval(a, env, tensors, consts) for a in e.args]
        if e.name in tensors:
            t = tensors[e.name]
            if len(args) != t.ndim:
                raise TcError("%s has %d dimensions, accessed with %d subscripts" % (e.name, t.ndim, len(args)))
            idx = []
            for d, a in enumerate(args):
                a = np.asarray(a)
                if a.dtype.kind not in "iu":
                    raise TcError("subscript %d of %s is not an integer" % (d, e.name))
                if a.size and (a.min() < 0 or a.max() >= t.shape[d]):
                    raise TcError("subscript %d of %s leaves [0, %d)" % (d, e.name, t.shape[d]))
                idx.append(a)
            return t[tuple(np.broadcast_arrays(*idx))] if idx else t[()]
        if e.name in _BUILTINS:
            return _BUILTINS[e.name](*[np.asarray(a, dtype=np.float64) for a in args])
        raise TcError("%s is neither a tensor nor a builtin" % e.name)
    raise TcError("cannot evaluate %r" % (e,))


_REDUCE = {"+": (np.add, 0.0), "*": (np.multiply, 1.0), "min": (np.minimum, np.inf), "max": (np.maximum, -np.inf)}


def run(func: Func, tensors: Dict[str, np.ndarray], scalars: Optional[Dict[str, object]] = None) -> Dict[str, np.ndarray]:
    """Evaluate the function on the given arguments; returns {output name: float64 array}.

    Floating-point tensors are widened to float64 (exactly), integer tensors to int64; every operation is done in
    float64 (subscripts in int64)."""
    plan = infer(func, {k: np.shape(v) for k, v in tensors.items()}, scalars)
    consts: Dict[str, object] = dict(plan.sizes)
    vals: Dict[str, np.ndarray] = {}
    for a in func.args:
        if a.shape is None:
            consts[a.name] = int(scalars[a.name]) if a.scalar_type in _INT_TYPES else float(scalars[a.name])
        else:
            arr = np.asarray(tensors[a.name])
            want_int = a.scalar_type in _INT_TYPES
            if want_int != (arr.dtype.kind in "iub"):
                raise TcError("%s is declared %s but holds %s" % (a.name, a.scalar_type, arr.dtype))
            vals[a.name] = arr.astype(np.int64 if want_int else np.float64)

    for st, rng in zip(func.stmts, plan.ranges):
        par = st.lhs_idx
        red = [v for v in rng if v not in par]
        order = par + red
        base = st.op.rstrip("!").rstrip("=")
        if st.op != "=" and not st.op.endswith("!") and st.lhs not in vals:
            raise TcError("%s accumulates onto %s, which holds nothing yet" % (st.op, st.lhs))
        if st.lhs not in vals:
            vals[st.lhs] = np.zeros(plan.shapes[st.lhs], dtype=np.float64)
        out = vals[st.lhs]
        extent = [rng[v][1] - rng[v][0] for v in order]
        if any(n <= 0 for n in extent[:len(par)]):
            continue  # an empty parallel range: nothing is assigned
        # The whole right-hand side is evaluated before anything is stored, slab by slab along the first index.
        result = np.empty(extent[:len(par)], dtype=np.float64)
        inner = int(np.prod(extent[1:], dtype=np.int64)) if len(extent) > 1 else 1
        step = max(1, _SLAB_ELEMS // max(inner, 1))
        lo0, hi0 = rng[order[0]] if order else (0, 1)
        for s0 in range(lo0, hi0, step):
            env, shape = {}, []
            for ax, v in enumerate(order):
                lo, hi = (s0, min(s0 + step, hi0)) if ax == 0 else rng[v]
                shp = [1] * len(order)
                shp[ax] = hi - lo
                env[v] = np.arange(lo, hi, dtype=np.int64).reshape(shp)
                shape.append(hi - lo)
            val = np.broadcast_to(np.asarray(_eval(st.rhs, env, vals, consts), dtype=np.float64), shape)
            if red:
                if any(n <= 0 for n in shape[len(par):]):
                    val = np.full(shape[:len(par)], _REDUCE[base][1])  # an empty reduction: the neutral element
                else:
                    val = _REDUCE[base][0].reduce(val.reshape(shape[:len(par)] + [-1]), axis=-1)
            if par:
                result[s0 - lo0:s0 - lo0 + shape[0]] = val
            else:
                result[()] = val
        where = tuple(slice(rng[v][0], rng[v][1]) for v in par)
        if st.op == "=" or st.op.endswith("!"):
            out[where] = result
        else:
            out[where] = _REDUCE[base][0](out[where], result)
    return {name: vals[name] for name in func.returns}


def output_shapes(text: str, arg_shapes: Dict[str, Tuple[int, ...]], scalars=None) -> Dict[str, Tuple[int, ...]]:
    """Shapes of the outputs of the function in `text` for arguments of the given shapes (range inference only)."""
    f = parse(text)
    plan = infer(f, arg_shapes, scalars)
    return {name: plan.shapes[name] for name in f.returns}


def evaluate(text: str, tensors: Dict[str, np.ndarray], scalars=None) -> Dict[str, np.ndarray]:
    """Parse and run in one call."""
    return run(parse(text), tensors, scalars)
