"""CPU oracle for the isolated per-partition training step and the coverage-corrected
gradient aggregation of gradient-only GNN training (Grappa).

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 numpy statement of what
the method computes, written from the paper's definitions, and exists only so that the
HIP implementation can be checked against it.  Nothing in the product package imports
it; only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may.  It shares no code, tables or helpers with the HIP path.

Modules
    graph      random (hash) node assignment and the isolated local subgraph   (design
               sections "Isolated Training Strategy" and "Graph Partitioning")
    gnn        GraphSAGE-mean / GCN / residual-GCN layers, weighted softmax
               cross-entropy and the hand-derived reverse pass                 (the
               model descriptions in the experimental setup; the true-gradient equation)
    gat        graph attention layers (one head) and their reverse pass              (the
               third model of the experimental setup)
    dropout    counter-based keep masks of the hidden layers                         (the
               hyper-parameters of the experimental setup)
    coverage   node-level weights, the minimum-distance factor, the shrinkage factor
               and the scale-then-reduce aggregation                           (section
               "Coverage-Corrected Aggregation"; the phase-parallel algorithm)
    sampling   isolated k-hop neighbour sampling inside the local subgraph
    step       glue: one partition's train step -> flat gradient + coverage statistics
    chunks     chunks, base + swept partitions, the sweep schedule and the switching
               controller                                                      (paragraph
               "Chunks and Efficient Partition Construction"; the controller subsection)
    optim      optimizer step (Adam / SGD) and the phase-parallel epoch loop          (the
               phase-parallel algorithm)

Pins (what each part is checked against, other than itself) live in
``tests/test_oracle_*.py``; a function with no independent pin says "parity unpinned"
in its docstring.
"""
