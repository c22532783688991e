"""CPU oracle for the BCR sparse product.  TEST INFRASTRUCTURE ONLY: imported
by tests/, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of
``bench.py``; never by the product package."""
