"""CPU oracle of the hot path.  Test infrastructure, not product code.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product package never does, and this
package never imports the product package.
"""
