"""MI355X task-graph mega-kernel decoder: Python binding over the C ABI in include/mpk.h."""
from .binding import *  # noqa: F401,F403
from .binding import lib, compile_graph, compile_set, compile_dag, Graph, GraphSet, Export, MpkError  # noqa: F401
