"""Developer tools: summarisers of rocprofv3 output (not imported by the library, the tests or bench.py)."""
